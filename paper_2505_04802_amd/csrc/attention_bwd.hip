// Gradient of tile-local multi-head self-attention (ORBIT-2 Sec. 4.2; the paper's
// headline numbers are training runs, Sec. 5).  The paper gives no formula of its
// own; this is the chain rule through  P = softmax(Q K^T / sqrt(dh)),  O = P V  for
// the tokens of one tile:
//     dV = P^T dO,   dP = dO V^T,   dS = P o (dP - delta),   delta_i = dO_i . O_i,
//     dQ = dS K / sqrt(dh),   dK = dS^T Q / sqrt(dh).
// P is never stored by the forward: it is recomputed here from Q, K and the
// log-sum-exp of every query that the forward returns.
//
// bf16 path = three launches, no atomics, deterministic:
//   1. attn_bwd_prep    delta_i per head (bandwidth-bound), written together with
//                       -lse_i*sqrt(dh) as 16-byte records (see below);
//   2. attn_bwd<KV=0>   query-stationary:  dQ;
//   3. attn_bwd<KV=1>   key-stationary:    dK and dV.
// Launches 2 and 3 are ONE kernel template.  As in the forward kernel a work unit is
// 128 "stationary" tokens of one (sample, tile, head), 32 per wave, kept in registers
// as MFMA B operands; the other side of the tile is streamed through LDS in blocks of
// BS tokens (global -> LDS directly, two stages).  Every product is computed
// transposed so that a lane owns one stationary token and the streamed index runs
// over the accumulator registers:
//     Sx  = Y1 X1^T      (stream x stationary)   Y1 = K | Q,   X1 = Q | K
//     dPx = Y2 X2^T                              Y2 = V | dO,  X2 = dO | V
//     P = exp2(c Sx - lse2),  dS = P o (dPx - delta)          (fp32, in registers)
//     acc1^T += Y1^T dS      (-> dQ^T | dK^T)     the accumulators of Sx/dPx are,
//     acc2^T += Y2^T P       (-> dV^T, KV only)   rounded to bf16, directly B operands
// Y1/Y2 are read from LDS twice: as 16-byte row fragments (A operand of the first
// pair of products) and through the transposing read ds_read_b64_tr_b16 (A operand
// of the second pair).  One XOR swizzle of the 16-byte chunks of a row keeps both
// access patterns free of bank conflicts.
//
// lse and delta belong to the QUERY.  Query-stationary: they are per-lane constants
// and enter as the initial value of the accumulator chains.  Key-stationary: the query
// is the register index, so they enter through one more MFMA step instead of 2 x 16
// per-register subtractions: the streamed block carries, per query, a 16-byte record
// with the value split into three bf16 summands (exact to 2^-24), multiplied by an
// all-ones B operand (lane half 0 feeds Sx, lane half 1 feeds dPx).
#include <type_traits>

#include "attention_common.h"

namespace reslim {

struct AttnBwdArgs {
  const bf16_t *qkv;     // [B, n_h, 3, heads, dh]
  const bf16_t *dout;    // [B, n_h, D]
  const u32x4 *aux;      // [2][B * heads * n_h] records: 0: -lse*sqrt(dh), 1: -delta; three bf16 summands + padding
  bf16_t *dqkv;          // [B, n_h, 3, heads, dh]
  const tile_desc *tiles;
  int T, heads, D, QB, total;
  int part;              // which 1/NSPLIT of the head's features this launch accumulates and writes
  int64_t n_h;
  int64_t aux_stride;    // records per array
  float c;               // MFMA output -> base-2 logit: log2(e) / sqrt(dh)   (1 when q is pre-scaled)
  float scq, sck;        // output factors of dQ and dK: 1 / sqrt(dh) both; with pre-scaled q dK takes ln 2
};

__device__ __forceinline__ u32x4 split3_bf16(float x) {
  const bf16_t h = f32_to_bf16(x);
  const float r1 = x - bf16_to_f32(h);
  const bf16_t m = f32_to_bf16(r1);
  const float r2 = r1 - bf16_to_f32(m);
  const bf16_t l = f32_to_bf16(r2);
  u32x4 o = {static_cast<uint32_t>(h) | (static_cast<uint32_t>(m) << 16), static_cast<uint32_t>(l), 0u, 0u};
  return o;
}
__device__ __forceinline__ float join3_bf16(uint32_t w0, uint32_t w1) {
  return bf16_to_f32(static_cast<bf16_t>(w0 & 0xffffu)) + bf16_to_f32(static_cast<bf16_t>(w0 >> 16)) +
         bf16_to_f32(static_cast<bf16_t>(w1 & 0xffffu));
}

// delta[b, head, tok] = sum over the head's features of dO * O; one thread per 8 features
template <int DH>
__global__ __launch_bounds__(256) void attn_bwd_prep_bf16_kernel(const bf16_t *out, const bf16_t *dout, const float *lse,
                                                                 u32x4 *aux, int64_t n_vec, int64_t n_h, int heads,
                                                                 int D, float lse_factor, int64_t aux_stride) {
  constexpr int LPH = DH / 8;   // lanes per head
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  const bool live = idx < n_vec;
  const int64_t i = live ? idx : 0;
  const u32x4 a = *reinterpret_cast<const u32x4 *>(out + i * 8);
  const u32x4 b = *reinterpret_cast<const u32x4 *>(dout + i * 8);
  float acc = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    acc = fmaf(__uint_as_float(a[e] << 16), __uint_as_float(b[e] << 16), acc);
    acc = fmaf(__uint_as_float(a[e] & 0xffff0000u), __uint_as_float(b[e] & 0xffff0000u), acc);
  }
#pragma unroll
  for (int w = 1; w < LPH; w <<= 1) acc += __shfl_xor(acc, w);
  const int vpr = D / 8;
  const int c8 = static_cast<int>(i % vpr);
  if (live && c8 % LPH == 0) {
    const int64_t row = i / vpr;
    const int head = c8 / LPH;
    const int64_t rec = (row / n_h * heads + head) * n_h + row % n_h;
    aux[rec] = split3_bf16(-lse[rec] * lse_factor);
    aux[aux_stride + rec] = split3_bf16(-acc);
  }
}

template <int OFF>
__device__ __forceinline__ uint64_t tr_issue(unsigned addr) {
  uint64_t r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}

// MODE: 0 = query-stationary, dQ;  1 = key-stationary, dK and dV;  2 = key-stationary, dV only;
// 3 = key-stationary, dK only (2 + 3 can replace 1 where the accumulators of both do not fit the
// register file next to the stationary fragments; no launch shape in use needs them).
// QS: q in qkv already carries the factor log2(e)/sqrt(dh) (as the fused QKV epilogue of the
// block leaves it): the MFMA output is the base-2 logit itself.
// NSPLIT: a launch accumulates only DH / NSPLIT of the head's output features (a.part says which)
// and recomputes the scores for each part; for heads whose full accumulators do not fit the
// register file next to the stationary fragments (dh = 256).
template <int DH, int BS, int MODE, bool QS, int MINW, int NST, int NSPLIT = 1>
__global__ __launch_bounds__(256, MINW) void attn_bwd_bf16_kernel(AttnBwdArgs a) {
  constexpr bool KV = MODE != 0;          // keys stationary
  constexpr bool DP = MODE != 2;          // dP = dO V^T is needed
  constexpr bool A1 = MODE != 2;          // accumulator 1: Y1^T dS  (dQ^T | dK^T)
  constexpr bool A2 = MODE == 1 || MODE == 2;   // accumulator 2: Y2^T P  (dV^T)
  constexpr int NW = 4;
  constexpr int BX = 32 * NW;             // stationary tokens per unit: 32 per wave
  constexpr int ROWB = DH * 2;
  constexpr int CPR = DH / 8;
  constexpr int RPB = 64 / CPR;
  constexpr int TILE_B = BS * ROWB;
  constexpr int AUXB = KV ? 2 * BS * 16 : 0;
  constexpr int AUXL = AUXB / 1024;       // wave-loads of the record block
  constexpr int STAGE = 2 * TILE_B + AUXB;
  constexpr int LPW = TILE_B / 1024 / NW;
  constexpr int NKT = BS / 32, NKS = DH / 16, NDT = DH / 32 / NSPLIT;   // NDT: 32-feature blocks of the accumulators
  constexpr bool PP = NKT == 2 && DH >= 128;   // wide heads with 64-token blocks: two groups in flight per wave
  constexpr bool HAND = DH <= 128;        // transposing reads issued by hand (see attention_common.h); needs a spill-free kernel
  static_assert(TILE_B % (1024 * NW) == 0 && AUXB % 1024 == 0 && NST * STAGE <= 160 * 1024, "LDS plan");
  static_assert((NST == 2 || NST == 3) && NKT <= 2, "ring of two or three stages of 32 or 64 tokens");
  extern __shared__ __align__(1024) unsigned char smem[];   // NST * STAGE bytes

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int l32 = lane & 31, hi = lane >> 5;
  const int ldq = 3 * a.D;
  const int ldx2 = KV ? ldq : a.D, ldy2 = KV ? a.D : ldq;
  const int G = gridDim.x;
  // chunk swizzle of a row, good for both the 16-byte row fragments (16 lanes, 16 rows, one
  // chunk column) and the transposing reads (32 lanes, 4 consecutive rows x 4 chunks)
  auto swz = [](int r) {
    return CPR == 8 ? ((((r >> 1) & 1) << 2) | (((r >> 2) & 1) << 1) | ((r >> 3) & 1)) : (((r & 3) << 2) | ((r >> 2) & 3));
  };

  // A unit = 128 stationary tokens of one (sample, tile, head); everything is uniform over the
  // work-group and kept as element offsets so that a descriptor costs few scalar registers.
  struct Unit {
    int n_t, r0, nsb;
    int64_t q_off;      // first element of the tile's q rows of this head in qkv / d_qkv
    int64_t o_off;      // ... of its rows in d_out
    int64_t aux_off;    // ... of its records in record array 0
  };
  auto decode = [&](int vb, Unit &u) -> int {      // first non-empty unit at or after vb (stride G), or >= total
    while (vb < a.total) {
      const int logical = xcd_remap_attn(vb, a.total);
      const int xb = logical % a.QB;
      int rest = logical / a.QB;
      const int head = rest % a.heads;
      rest /= a.heads;
      const int tile = rest % a.T;
      const int b = rest / a.T;
      const int n_t = a.tiles[tile].n_tok;
      if (xb * BX < n_t) {
        const int64_t row0 = static_cast<int64_t>(b) * a.n_h + a.tiles[tile].tok_off;
        u.n_t = n_t;
        u.r0 = xb * BX;
        u.nsb = (n_t + BS - 1) / BS;
        u.q_off = row0 * ldq + head * DH;
        u.o_off = row0 * a.D + head * DH;
        u.aux_off = (static_cast<int64_t>(b) * a.heads + head) * a.n_h + a.tiles[tile].tok_off;
        return vb;
      }
      vb += G;
    }
    return vb;
  };
  auto x1_of = [&](const Unit &u) { return a.qkv + u.q_off + (KV ? a.D : 0); };
  auto x2_of = [&](const Unit &u) { return KV ? a.qkv + u.q_off + 2 * a.D : a.dout + u.o_off; };
  auto y1_of = [&](const Unit &u) { return a.qkv + u.q_off + (KV ? 0 : a.D); };
  auto y2_of = [&](const Unit &u) { return KV ? a.dout + u.o_off : a.qkv + u.q_off + 2 * a.D; };
  Unit cur, nxt;
  int vb = decode(blockIdx.x, cur);
  if (vb >= a.total) return;
  // the loads run NST - 1 blocks ahead of the arithmetic, across unit boundaries: a second
  // cursor walks the same sequence of (unit, block)
  Unit iu = cur;
  int ivb = vb, iblk = 0;
  vb = decode(vb + G, nxt);
  bool has_next = vb < a.total;

  // ---- load side: lane -> (row of the block, 16-byte chunk), per-lane byte offsets
  int ld_row[LPW], off1[LPW], off2[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    ld_row[i] = (wave + NW * i) * RPB + lane / CPR;
    const int ch = ((lane % CPR) ^ swz(ld_row[i])) * 16;
    off1[i] = ld_row[i] * ldq * 2 + ch;
    off2[i] = ld_row[i] * ldy2 * 2 + ch;
  }
  const int aux_L = wave * 64 + lane;                 // record slot of this lane in the block (KV only)
  const int aux_arr = aux_L / BS, aux_row = aux_L % BS;
  auto issue = [&](const Unit &u, int s0, int buf) {
    unsigned char *sb = smem + buf * STAGE;
    const unsigned char *g1 = reinterpret_cast<const unsigned char *>(y1_of(u) + static_cast<size_t>(s0) * ldq);
    const unsigned char *g2 = reinterpret_cast<const unsigned char *>(y2_of(u) + static_cast<size_t>(s0) * ldy2);
    const int lim = u.n_t - 1 - s0;       // last valid row of this block
    if (lim >= BS - 1) {                   // whole block inside the tile (uniform)
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        attn_dl_load16(reinterpret_cast<const bf16_t *>(g1 + static_cast<uint32_t>(off1[i])), sb + (wave + NW * i) * 1024);
        attn_dl_load16(reinterpret_cast<const bf16_t *>(g2 + static_cast<uint32_t>(off2[i])),
                       sb + TILE_B + (wave + NW * i) * 1024);
      }
    } else {                               // rows past the tile end re-read its last row (finite; masked later)
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        const int back = max(ld_row[i] - lim, 0);
        attn_dl_load16(reinterpret_cast<const bf16_t *>(g1 + static_cast<uint32_t>(off1[i] - back * ldq * 2)),
                       sb + (wave + NW * i) * 1024);
        attn_dl_load16(reinterpret_cast<const bf16_t *>(g2 + static_cast<uint32_t>(off2[i] - back * ldy2 * 2)),
                       sb + TILE_B + (wave + NW * i) * 1024);
      }
    }
    if constexpr (KV) {
      if (wave < AUXL) {
        const int row = s0 + min(aux_row, lim);
        attn_dl_load16(reinterpret_cast<const bf16_t *>(a.aux + u.aux_off + aux_arr * a.aux_stride + row),
                       sb + 2 * TILE_B + wave * 1024);
      }
    }
  };
  bf16x8 x1f[NKS], x2f[DP ? NKS : 1];
  f32x16 sinit, dpinit;
  auto load_x = [&](const Unit &u) {
    const int xrow = min(u.r0 + wave * 32 + l32, u.n_t - 1);
    const bf16_t *p1 = x1_of(u) + static_cast<size_t>(xrow) * ldq + hi * 8;
    const bf16_t *p2 = x2_of(u) + static_cast<size_t>(xrow) * ldx2 + hi * 8;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      x1f[ks] = *reinterpret_cast<const bf16x8 *>(p1 + ks * 16);
      if constexpr (DP) x2f[ks] = *reinterpret_cast<const bf16x8 *>(p2 + ks * 16);
    }
    float si = 0.f, di = 0.f;
    if constexpr (!KV) {
      const u32x2 r0 = *reinterpret_cast<const u32x2 *>(a.aux + u.aux_off + xrow);
      const u32x2 r1 = *reinterpret_cast<const u32x2 *>(a.aux + u.aux_off + a.aux_stride + xrow);
      si = join3_bf16(r0[0], r0[1]);
      di = join3_bf16(r1[0], r1[1]);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) { sinit[r] = si; dpinit[r] = di; }
  };

  // ---- read side
  // Row fragment: A-operand row l32 carries streamed token key_perm(l32) of its 32-token group.
  // Transposed fragment: this lane points at token row 8*hi + 4*e + (lane%16)/4 of a 16-token
  // step and at the 4 features 32*d + 16*((lane/16)&1) + 4*(lane%4) .. +3.
  const int yr = key_perm(l32);
  const int y_row = yr * ROWB, y_swz = swz(yr);
  const int L16 = lane & 15;
  int t_addr[2][NDT];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int vr = 8 * hi + 4 * e + (L16 >> 2);
#pragma unroll
    for (int d = 0; d < NDT; ++d) {
      const int o = 32 * (d + a.part * NDT) + 16 * ((lane >> 4) & 1) + 4 * (L16 & 3);
      t_addr[e][d] = vr * ROWB + (((o >> 3) ^ swz(vr)) << 4) + ((o >> 2) & 1) * 8;
    }
  }
  const int aux_addr = 2 * TILE_B + hi * BS * 16 + yr * 16;

  // all-ones B operands of the record step: lane half 0 -> Sx, lane half 1 -> dPx
  bf16x8 ones_s, ones_d;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    ones_s[e] = static_cast<__bf16>(e < 3 && hi == 0 ? 1.0f : 0.0f);
    ones_d[e] = static_cast<__bf16>(e < 3 && hi == 1 ? 1.0f : 0.0f);
  }

  f32x16 acc1[A1 ? NDT : 1], acc2[A2 ? NDT : 1];
  auto reset = [&]() {
#pragma unroll
    for (int d = 0; d < (A1 ? NDT : 1); ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc1[d][r] = 0.f;
#pragma unroll
    for (int d = 0; d < (A2 ? NDT : 1); ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc2[d][r] = 0.f;
  };
  reset();
  load_x(cur);
  // issue the next block of the load cursor into stage `buf`; false when the sequence has ended
  auto issue_next = [&](int buf) -> bool {
    if (ivb >= a.total) return false;
    issue(iu, iblk * BS, buf);
    if (++iblk == iu.nsb) {
      ivb = decode(ivb + G, iu);
      iblk = 0;
    }
    return true;
  };
  // The same in two steps, for the kernels that keep two groups in flight: plan_next() picks the
  // block and moves the cursor, issue_part(i) sends this wave's i-th pair of direct loads (the
  // record load rides with pair 0).  A wave's burst of loads stalls it while the CU's load queue
  // is full; spread between the MFMAs of the first score product they cost nothing.  Blocks that
  // cross the tile end, and waves without stationary tokens, keep the burst.
  struct Pending {
    const unsigned char *g1, *g2;
    const u32x4 *aux;
    unsigned char *sb;
    int lim;
  } pend;
  auto plan_next = [&](int buf) -> bool {
    if (ivb >= a.total) return false;
    const int s0 = iblk * BS;
    pend.sb = smem + buf * STAGE;
    pend.g1 = reinterpret_cast<const unsigned char *>(y1_of(iu) + static_cast<size_t>(s0) * ldq);
    pend.g2 = reinterpret_cast<const unsigned char *>(y2_of(iu) + static_cast<size_t>(s0) * ldy2);
    pend.aux = a.aux + iu.aux_off + s0;
    pend.lim = iu.n_t - 1 - s0;
    if (++iblk == iu.nsb) {
      ivb = decode(ivb + G, iu);
      iblk = 0;
    }
    return true;
  };
  auto issue_part = [&](int i) {          // only for blocks wholly inside the tile
    attn_dl_load16(reinterpret_cast<const bf16_t *>(pend.g1 + static_cast<uint32_t>(off1[i])), pend.sb + (wave + NW * i) * 1024);
    attn_dl_load16(reinterpret_cast<const bf16_t *>(pend.g2 + static_cast<uint32_t>(off2[i])),
                   pend.sb + TILE_B + (wave + NW * i) * 1024);
    if constexpr (KV) {
      if (i == 0 && wave < AUXL)
        attn_dl_load16(reinterpret_cast<const bf16_t *>(pend.aux + aux_arr * a.aux_stride + aux_row),
                       pend.sb + 2 * TILE_B + wave * 1024);
    }
  };
  auto issue_planned_burst = [&]() {      // any block: rows past the tile end re-read its last row
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      const int back = max(ld_row[i] - pend.lim, 0);
      attn_dl_load16(reinterpret_cast<const bf16_t *>(pend.g1 + static_cast<uint32_t>(off1[i] - back * ldq * 2)),
                     pend.sb + (wave + NW * i) * 1024);
      attn_dl_load16(reinterpret_cast<const bf16_t *>(pend.g2 + static_cast<uint32_t>(off2[i] - back * ldy2 * 2)),
                     pend.sb + TILE_B + (wave + NW * i) * 1024);
    }
    if constexpr (KV) {
      if (wave < AUXL)
        attn_dl_load16(reinterpret_cast<const bf16_t *>(pend.aux + aux_arr * a.aux_stride + min(aux_row, pend.lim)),
                       pend.sb + 2 * TILE_B + wave * 1024);
    }
  };
  constexpr int NLD = 2 * LPW;            // direct loads of one block per wave (+1 in the waves that fetch records)
  int ahead = 0;                          // blocks in flight beyond the one about to be computed
  issue_next(0);
#pragma unroll
  for (int i = 1; i < NST - 1; ++i) ahead += issue_next(i) ? 1 : 0;

  int sb = 0, buf = 0;
  for (;;) {
    // block `sb` of `cur` must have landed; younger blocks may stay in flight.  Loads complete in
    // issue order, so "at most `ahead` blocks' worth outstanding" is enough.
    if (NST == 2 || ahead == 0) {
      __builtin_amdgcn_s_waitcnt(0x0F70);
    } else if (KV && wave < AUXL) {
      __builtin_amdgcn_s_waitcnt(0x0F70 | ((NLD + 1) & 15) | (((NLD + 1) >> 4) << 14));
    } else {
      __builtin_amdgcn_s_waitcnt(0x0F70 | (NLD & 15) | ((NLD >> 4) << 14));
    }
    // a bare barrier: __syncthreads() would add a fence that waits for ALL vector-memory operations,
    // the younger prefetches included.  Every wave has waited for its own direct-to-LDS loads of
    // this block above, and LDS reads of the stage being refilled finished before its readers arrived.
    __builtin_amdgcn_s_barrier();           // everybody's part of the block is in LDS; the oldest stage is free
    const bool last = sb + 1 == cur.nsb;
    const bool active = cur.r0 + wave * 32 < cur.n_t;
    bool spread = false;                    // this wave sends the next block's loads between its MFMAs
    {
      int ibuf = buf + NST - 1;
      if (ibuf >= NST) ibuf -= NST;
      bool issued;
      if constexpr (PP) {
        issued = plan_next(ibuf);
        spread = issued && active && pend.lim >= BS - 1;
        if (issued && !spread) issue_planned_burst();
      } else {
        issued = issue_next(ibuf);
      }
      if (issued) { if (NST == 2) ahead = 0; }   // one computed, one issued: `ahead` unchanged
      else if (ahead > 0) --ahead;
    }
    const unsigned char *st = smem + buf * STAGE;
    const int s0 = sb * BS;

    // The work on one 32-token group of the streamed block, in three phases.
    const unsigned st_off = static_cast<unsigned>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) const unsigned char *)st));
    // `between(i)`, i < 16: vector work of ANOTHER group placed behind the MFMAs of this one, so
    // that one wave keeps both pipes busy (wide heads run a single wave per SIMD)
    auto scores = [&](auto kt_c, f32x16 &s, f32x16 &dp, auto between) {          // matrix pipe
      constexpr int kt = decltype(kt_c)::value;
      if constexpr (DH >= 128) {
        // wide heads: the fragment reads run PF steps ahead of the MFMAs that use them, in a ring
        // of PF + 1 register sets, and a scheduling barrier per step keeps that order (left to
        // itself the compiler either waits for every read right before its MFMA or hoists all
        // reads of the group to its top: 64+ registers of fragments next to the accumulators)
        constexpr int PF = 2;
        bf16x8 f1[PF + 1], f2[DP ? PF + 1 : 1];
        auto fetch = [&](int ks) {
          const unsigned char *rp = st + kt * 32 * ROWB + y_row + (((2 * ks + hi) ^ y_swz) << 4);
          f1[ks % (PF + 1)] = *reinterpret_cast<const bf16x8 *>(rp);
          if constexpr (DP) f2[ks % (PF + 1)] = *reinterpret_cast<const bf16x8 *>(rp + TILE_B);
        };
#pragma unroll
        for (int ks = 0; ks < PF; ++ks) fetch(ks);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          if (ks + PF < NKS) fetch(ks + PF);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1[ks % (PF + 1)], x1f[ks], ks == 0 ? sinit : s, 0, 0, 0);
          if constexpr (DP) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2[ks % (PF + 1)], x2f[ks], ks == 0 ? dpinit : dp, 0, 0, 0);
#pragma unroll
          for (int i = ks * 16 / NKS; i < (ks + 1) * 16 / NKS; ++i) between(i);
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          const unsigned char *rp = st + kt * 32 * ROWB + y_row + (((2 * ks + hi) ^ y_swz) << 4);
          const bf16x8 f1 = *reinterpret_cast<const bf16x8 *>(rp);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1, x1f[ks], ks == 0 ? sinit : s, 0, 0, 0);
          if constexpr (DP) {
            const bf16x8 f2 = *reinterpret_cast<const bf16x8 *>(rp + TILE_B);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2, x2f[ks], ks == 0 ? dpinit : dp, 0, 0, 0);
          }
#pragma unroll
          for (int i = ks * 16 / NKS; i < (ks + 1) * 16 / NKS; ++i) between(i);
        }
      }
      if constexpr (KV) {
        const bf16x8 fa = *reinterpret_cast<const bf16x8 *>(st + aux_addr + kt * 32 * 16);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, ones_s, s, 0, 0, 0);
        if constexpr (DP) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, ones_d, dp, 0, 0, 0);
      }
    };
    auto mask = [&](int kt, f32x16 &s) {      // ragged end: streamed tokens past the tile end get probability 0
      if (s0 + kt * 32 + 32 > cur.n_t) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = s0 + kt * 32 + 16 * (r / 8) + 8 * hi + (r % 8);
          if (row >= cur.n_t) s[r] = -INFINITY;
        }
      }
    };
    auto prob1 = [&](f32x16 &s, f32x16 &dp, int r) {                // vector pipe: s <- P, dp <- dS
      s[r] = __builtin_amdgcn_exp2f(QS ? s[r] : s[r] * a.c);
      if constexpr (DP) dp[r] *= s[r];
    };
    auto probs = [&](f32x16 &s, f32x16 &dp) {
#pragma unroll
      for (int r = 0; r < 16; ++r) prob1(s, dp, r);
    };
    auto nothing = [](int) {};
    auto products = [&](auto kt_c, const f32x16 &s, const f32x16 &dp, auto between) {   // matrix pipe
      constexpr int kt = decltype(kt_c)::value;
      auto step = [&](auto h2_c) {
        constexpr int h2 = decltype(h2_c)::value;
        constexpr int ROFF = (kt * 32 + h2 * 16) * ROWB;
        bf16x8 pf, dsf;
        typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
        if constexpr (HAND) {
          uint64_t r1[NDT][2], r2[NDT][2];
#pragma unroll
          for (int d = 0; d < NDT; ++d)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              if constexpr (A1) r1[d][e] = tr_issue<ROFF>(st_off + static_cast<unsigned>(t_addr[e][d]));
              if constexpr (A2) r2[d][e] = tr_issue<ROFF + TILE_B>(st_off + static_cast<unsigned>(t_addr[e][d]));
            }
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            if constexpr (A1) dsf[e] = static_cast<__bf16>(dp[8 * h2 + e]);
            if constexpr (A2) pf[e] = static_cast<__bf16>(s[8 * h2 + e]);
          }
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
          for (int d = 0; d < NDT; ++d)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              if constexpr (A1) asm volatile("" : "+v"(r1[d][e]));
              if constexpr (A2) asm volatile("" : "+v"(r2[d][e]));
            }
#pragma unroll
          for (int d = 0; d < NDT; ++d) {
            if constexpr (A1) {
              const u64x2 b1 = {r1[d][0], r1[d][1]};
              acc1[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b1), dsf, acc1[d], 0, 0, 0);
            }
            if constexpr (A2) {
              const u64x2 b2 = {r2[d][0], r2[d][1]};
              acc2[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b2), pf, acc2[d], 0, 0, 0);
            }
#pragma unroll
            for (int i = (h2 * NDT + d) * 8 / NDT; i < (h2 * NDT + d + 1) * 8 / NDT; ++i) between(i);
          }
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            if constexpr (A1) dsf[e] = static_cast<__bf16>(dp[8 * h2 + e]);
            if constexpr (A2) pf[e] = static_cast<__bf16>(s[8 * h2 + e]);
          }
          typedef __attribute__((ext_vector_type(8))) short s16x8;
          auto tr_frag = [&](int off) {
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3))) *)(st + off));
            return lo;
          };
#pragma unroll
          for (int d = 0; d < NDT; ++d) {
            if constexpr (A1) {
              const s16x8 both = __builtin_shufflevector(tr_frag(ROFF + t_addr[0][d]), tr_frag(ROFF + t_addr[1][d]), 0, 1, 2, 3, 4, 5, 6, 7);
              acc1[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), dsf, acc1[d], 0, 0, 0);
            }
            if constexpr (A2) {
              const s16x8 both = __builtin_shufflevector(tr_frag(ROFF + TILE_B + t_addr[0][d]), tr_frag(ROFF + TILE_B + t_addr[1][d]), 0, 1, 2, 3, 4, 5, 6, 7);
              acc2[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), pf, acc2[d], 0, 0, 0);
            }
#pragma unroll
            for (int i = (h2 * NDT + d) * 8 / NDT; i < (h2 * NDT + d + 1) * 8 / NDT; ++i) between(i);
          }
        }
      };
      step(std::integral_constant<int, 0>{});
      step(std::integral_constant<int, 1>{});
    };
    // One straight path for every block, one 32-token group after the other; a second group
    // that lies wholly past the tile end (last block only) is computed and masked to zero rather
    // than skipped.  The next unit's stationary fragments are fetched at ONE place, after the
    // last scores that use the current ones.
    const bool ragged = s0 + BS > cur.n_t;
    f32x16 sA, dA;
    if constexpr (PP) {
      // two groups in flight: the exponentials of one sit between the MFMAs of the other
      f32x16 sB, dB;
      if (active) {
        scores(std::integral_constant<int, 0>{}, sA, dA, [&](int i) {
          if (spread && i % (16 / LPW) == 0) issue_part(i / (16 / LPW));
        });
        if (ragged) mask(0, sA);
        scores(std::integral_constant<int, 1>{}, sB, dB, [&](int i) { prob1(sA, dA, i); });
      }
      if (last && has_next) load_x(nxt);
      if (active) {
        if (ragged) mask(1, sB);
        products(std::integral_constant<int, 0>{}, sA, dA, [&](int i) { prob1(sB, dB, i); });
        products(std::integral_constant<int, 1>{}, sB, dB, nothing);
      }
    } else {
      if constexpr (NKT == 2) {
        if (active) {
          scores(std::integral_constant<int, 0>{}, sA, dA, nothing);
          if (ragged) mask(0, sA);
          probs(sA, dA);
          products(std::integral_constant<int, 0>{}, sA, dA, nothing);
        }
      }
      if (active) scores(std::integral_constant<int, NKT - 1>{}, sA, dA, nothing);
      if (last && has_next) load_x(nxt);
      if (active) {
        if (ragged) mask(NKT - 1, sA);
        probs(sA, dA);
        products(std::integral_constant<int, NKT - 1>{}, sA, dA, nothing);
      }
    }
    if (++buf == NST) buf = 0;
    if (!last) { ++sb; continue; }

    // ---- end of a unit: scale, round and store this lane's row of each gradient
    const int xrow = cur.r0 + wave * 32 + l32;
    if (active && xrow < cur.n_t) {
      bf16_t *p1 = a.dqkv + cur.q_off + (KV ? a.D : 0) + static_cast<size_t>(xrow) * ldq + hi * 4 + a.part * NDT * 32;
      bf16_t *p2 = a.dqkv + cur.q_off + 2 * a.D + static_cast<size_t>(xrow) * ldq + hi * 4 + a.part * NDT * 32;
      const float sc1 = KV ? a.sck : a.scq;
#pragma unroll
      for (int d = 0; d < NDT; ++d)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          // registers 4*r4 .. 4*r4+3 hold features 32d + 8*r4 + 4*hi + (0..3) of this lane's token
          bf16x4 tmp;
          if constexpr (A1) {
#pragma unroll
            for (int e = 0; e < 4; ++e) tmp[e] = static_cast<__bf16>(acc1[d][4 * r4 + e] * sc1);
            *reinterpret_cast<u32x2 *>(p1 + d * 32 + r4 * 8) = __builtin_bit_cast(u32x2, tmp);
          }
          if constexpr (A2) {
#pragma unroll
            for (int e = 0; e < 4; ++e) tmp[e] = static_cast<__bf16>(acc2[d][4 * r4 + e]);
            *reinterpret_cast<u32x2 *>(p2 + d * 32 + r4 * 8) = __builtin_bit_cast(u32x2, tmp);
          }
        }
    }
    if (!has_next) break;
    // Everything in flight (the next unit's stationary fragments, the result stores, the
    // prefetched blocks) is waited for here, once per unit: with register loads possibly
    // pending across the loop edge the compiler would otherwise wait for ALL vector-memory
    // operations, the prefetch included, before the first fragment use of every block.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    cur = nxt;
    vb = decode(vb + G, nxt);
    has_next = vb < a.total;
    sb = 0;
    reset();
  }
}

// ------------------------------------------------------------------ fp32 debug path
__global__ __launch_bounds__(256) void attn_bwd_delta_f32_kernel(const float *out, const float *dout, float *delta,
                                                                 int64_t n, int64_t n_h, int heads, int dh) {
  // one thread per (sample, token, head)
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= n) return;
  const int head = static_cast<int>(idx % heads);
  const int64_t row = idx / heads;
  const float *o = out + (row * heads + head) * dh;
  const float *d_o = dout + (row * heads + head) * dh;
  float acc = 0.f;
  for (int d = 0; d < dh; ++d) acc = fmaf(o[d], d_o[d], acc);
  delta[(row / n_h * heads + head) * n_h + row % n_h] = acc;
}

// KV = false: one work-group per query token, gradient of q.  KV = true: one per key token, gradients of k and v.
template <bool KV>
__global__ __launch_bounds__(128) void attn_bwd_f32_kernel(const float *qkv, const float *dout, const float *lse,
                                                           const float *delta, float *dqkv, const tile_desc *tiles,
                                                           const int32_t *tile_of_tok, int64_t n_h, int heads, int D,
                                                           int dh, int max_n_tok) {
  extern __shared__ float sm[];
  float *wds = sm;                      // [max_n_tok] dS towards every token of the other side
  float *wp = sm + max_n_tok;           // [max_n_tok] P (KV only)
  float *x1 = sm + 2 * max_n_tok;       // [dh] this token's q (or k)
  float *x2 = x1 + dh;                  // [dh] this token's dO (or v)
  const int64_t tok = blockIdx.x;
  const int head = blockIdx.y, b = blockIdx.z;
  const int tile = tile_of_tok[tok];
  const int n_t = tiles[tile].n_tok;
  const int64_t tok_off = tiles[tile].tok_off;
  const int ld = 3 * D;
  const size_t row_b = static_cast<size_t>(b) * n_h;
  const float *qb = qkv + (row_b + tok_off) * ld + head * dh;             // q of the tile's first token
  const float *dob = dout + (row_b + tok_off) * D + head * dh;
  const float *stat = lse + (static_cast<size_t>(b) * heads + head) * n_h;
  const float *dstat = delta + (static_cast<size_t>(b) * heads + head) * n_h;
  const float *mine = qkv + (row_b + tok) * ld + head * dh;
  const int t = threadIdx.x;
  for (int d = t; d < dh; d += 128) {
    x1[d] = KV ? mine[D + d] : mine[d];
    x2[d] = KV ? mine[2 * D + d] : dout[(row_b + tok) * D + head * dh + d];
  }
  __syncthreads();
  const float scale = rsqrtf(static_cast<float>(dh));
  for (int j = t; j < n_t; j += 128) {
    // KV: j is a query, this token the key; else j is a key, this token the query
    const float *y1 = qb + static_cast<size_t>(j) * ld + (KV ? 0 : D);
    const float *y2 = KV ? dob + static_cast<size_t>(j) * D : qb + static_cast<size_t>(j) * ld + 2 * D;
    float s = 0.f, dp = 0.f;
    for (int d = 0; d < dh; ++d) {
      s = fmaf(x1[d], y1[d], s);
      dp = fmaf(x2[d], y2[d], dp);
    }
    const int64_t qi = KV ? tok_off + j : tok;
    const float p = expf(s * scale - stat[qi]);
    wds[j] = p * (dp - dstat[qi]);
    if (KV) wp[j] = p;
  }
  __syncthreads();
  float *go = dqkv + (row_b + tok) * ld + head * dh;
  for (int d = t; d < dh; d += 128) {
    float a1 = 0.f, a2 = 0.f;
    for (int j = 0; j < n_t; ++j) {
      a1 = fmaf(wds[j], qb[static_cast<size_t>(j) * ld + (KV ? 0 : D) + d], a1);
      if (KV) a2 = fmaf(wp[j], dob[static_cast<size_t>(j) * D + d], a2);
    }
    if (KV) {
      go[D + d] = a1 * scale;
      go[2 * D + d] = a2;
    } else {
      go[d] = a1 * scale;
    }
  }
}

template <int DH, int BS, int NST>
constexpr int bwd_lds_bytes(bool kv) { return NST * (2 * BS * DH * 2 + (kv ? 2 * BS * 16 : 0)); }

static int g_bwd_cus = 0;
static bool g_bwd_big_ok = false;

hipError_t attention_bwd_init() {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&g_bwd_cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  // kernels whose LDS ring exceeds the default limit of a launch (64 KiB)
  g_bwd_big_ok = true;
  struct Big { const void *fn; int bytes; };
  const Big big[] = {
#define RESLIM_BIG(DH, BS, MODE, NST, NSPLIT)                                                                       \
  {reinterpret_cast<const void *>(&attn_bwd_bf16_kernel<DH, BS, MODE, false, 1, NST, NSPLIT>), bwd_lds_bytes<DH, BS, NST>(MODE != 0)}, \
  {reinterpret_cast<const void *>(&attn_bwd_bf16_kernel<DH, BS, MODE, true, 1, NST, NSPLIT>), bwd_lds_bytes<DH, BS, NST>(MODE != 0)},
      RESLIM_BIG(128, 64, 0, 3, 1) RESLIM_BIG(128, 64, 3, 3, 1) RESLIM_BIG(128, 64, 1, 3, 1)
      RESLIM_BIG(256, 32, 0, 3, 1) RESLIM_BIG(256, 32, 1, 3, 2)
#undef RESLIM_BIG
  };
  for (const Big &k : big) {
    e = hipFuncSetAttribute(k.fn, hipFuncAttributeMaxDynamicSharedMemorySize, k.bytes);
    if (e != hipSuccess) {            // not fatal: only the gradient at head dimensions 128 and 256 is refused
      (void)hipGetLastError();
      g_bwd_big_ok = false;
    }
  }
  return hipSuccess;
}

size_t tiles_attention_bwd_ws_bytes(const reslim_ctx *c, int batch, const SeqGeom *geom) {
  const size_t recs = static_cast<size_t>(batch) * c->cfg.heads * (geom ? geom->n_h : c->n_h);
  return c->cfg.dtype == RESLIM_BF16 ? align256(recs * 32) : align256(recs * 4);
}

template <int DH, int BS, int MODE, bool QS, int MINW, int NST, int NSPLIT = 1>
static hipError_t launch_bwd_one(const AttnBwdArgs &a0, hipStream_t st) {
  const int g = a0.total < MINW * g_bwd_cus ? a0.total : MINW * g_bwd_cus;    // persistent grid
  AttnBwdArgs a = a0;
  for (a.part = 0; a.part < NSPLIT; ++a.part) {
    attn_bwd_bf16_kernel<DH, BS, MODE, QS, MINW, NST, NSPLIT><<<dim3(g), dim3(256), bwd_lds_bytes<DH, BS, NST>(MODE != 0), st>>>(a);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// Launch shapes (measured on MI355X; the file is built with MFMA operands in ordinary vector
// registers, see the build script): dh = 64: 64-token blocks, three stages; the dQ kernel fits 168
// registers = three work-groups per CU, the dK/dV kernel (197) two.  dh = 128: one work-group per
// CU, 64-token blocks with two 32-token groups in flight; dQ ~350 registers, dK and dV together
// ~510, no spills (c4: 7.1 ms; 13.1 ms with 32-token blocks, separate dK and dV passes and
// accumulator-register MFMAs; 17.4 ms with two spilling work-groups).  dh = 256: dQ unsplit on
// 32-token blocks (15 registers spilled, still faster than two spill-free half passes), dK and dV
// together, once per half of the head's features (505 registers, no spills).  The 10B model's
// block: 6.6 ms, against 40.5 ms for unsplit dQ and dK/dV passes that spilled 130 .. 145 registers.
template <bool QS>
static hipError_t launch_bwd_all(const AttnBwdArgs &a, int dh, hipStream_t st) {
  hipError_t e;
  switch (dh) {
    case 64:
      e = launch_bwd_one<64, 64, 0, QS, 3, 3>(a, st);
      return e != hipSuccess ? e : launch_bwd_one<64, 64, 1, QS, 2, 3>(a, st);
    case 128:
      if (!g_bwd_big_ok) return hipErrorInvalidValue;
      e = launch_bwd_one<128, 64, 0, QS, 1, 3>(a, st);
      return e != hipSuccess ? e : launch_bwd_one<128, 64, 1, QS, 1, 3>(a, st);
    case 256:
      if (!g_bwd_big_ok) return hipErrorInvalidValue;
      e = launch_bwd_one<256, 32, 0, QS, 1, 3, 1>(a, st);
      return e != hipSuccess ? e : launch_bwd_one<256, 32, 1, QS, 1, 3, 2>(a, st);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_tiles_attention_bwd(const reslim_ctx *c, const void *qkv, const void *out, const float *lse,
                                      const void *dout, void *dqkv, int batch, void *ws, bool q_prescaled,
                                      hipStream_t st, const SeqGeom *geom) {
  const SeqGeom sg = geom ? *geom : ctx_geom(c);
  const int heads = c->cfg.heads, D = c->cfg.embed_dim, dh = c->dh;
  const int64_t recs = static_cast<int64_t>(batch) * heads * sg.n_h;
  if (recs == 0) return hipSuccess;
  if (c->cfg.dtype == RESLIM_BF16) {
    const float rs = 1.0f / sqrtf(static_cast<float>(dh));
    AttnBwdArgs a;
    a.qkv = static_cast<const bf16_t *>(qkv);
    a.dout = static_cast<const bf16_t *>(dout);
    a.aux = static_cast<const u32x4 *>(ws);
    a.dqkv = static_cast<bf16_t *>(dqkv);
    a.tiles = sg.d_tiles;
    a.T = sg.T;
    a.heads = heads;
    a.D = D;
    a.n_h = sg.n_h;
    a.aux_stride = recs;
    // With q pre-scaled by log2(e)/sqrt(dh) the MFMA output is the base-2 logit; the gradient with
    // respect to the UNSCALED q keeps the factor 1/sqrt(dh), the one of k becomes ln 2 (k meets the
    // scaled q).
    a.c = q_prescaled ? 1.0f : 1.4426950408889634f * rs;
    a.scq = rs;
    a.sck = q_prescaled ? 0.69314718055994531f : rs;
    a.QB = (sg.max_n_tok + 127) / 128;
    const int64_t total = static_cast<int64_t>(batch) * sg.T * heads * a.QB;
    if (total > INT32_MAX || g_bwd_cus <= 0) return hipErrorInvalidValue;
    a.total = static_cast<int>(total);
    const int64_t n_vec = static_cast<int64_t>(batch) * sg.n_h * D / 8;
    const unsigned pg = static_cast<unsigned>((n_vec + 255) / 256);
    // record 0 holds -lse in the unit of the MFMA output: -lse*sqrt(dh), or -lse*log2(e) for pre-scaled q
    const float lse_f = q_prescaled ? 1.4426950408889634f : sqrtf(static_cast<float>(dh));
    u32x4 *aux = static_cast<u32x4 *>(ws);
    const bf16_t *o = static_cast<const bf16_t *>(out);
    switch (dh) {
      case 64: attn_bwd_prep_bf16_kernel<64><<<dim3(pg), dim3(256), 0, st>>>(o, a.dout, lse, aux, n_vec, sg.n_h, heads, D, lse_f, recs); break;
      case 128: attn_bwd_prep_bf16_kernel<128><<<dim3(pg), dim3(256), 0, st>>>(o, a.dout, lse, aux, n_vec, sg.n_h, heads, D, lse_f, recs); break;
      case 256: attn_bwd_prep_bf16_kernel<256><<<dim3(pg), dim3(256), 0, st>>>(o, a.dout, lse, aux, n_vec, sg.n_h, heads, D, lse_f, recs); break;
      default: return hipErrorInvalidValue;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return q_prescaled ? launch_bwd_all<true>(a, dh, st) : launch_bwd_all<false>(a, dh, st);
  }
  float *delta = static_cast<float *>(ws);
  const size_t lds = (2 * static_cast<size_t>(sg.max_n_tok) + 2 * dh) * sizeof(float);
  if (lds > 60 * 1024 || sg.n_h > INT32_MAX) return hipErrorInvalidValue;
  const int64_t n = static_cast<int64_t>(batch) * sg.n_h * heads;
  attn_bwd_delta_f32_kernel<<<dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st>>>(
      static_cast<const float *>(out), static_cast<const float *>(dout), delta, n, sg.n_h, heads, dh);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid(static_cast<unsigned>(sg.n_h), heads, batch);
  attn_bwd_f32_kernel<false><<<grid, dim3(128), lds, st>>>(static_cast<const float *>(qkv), static_cast<const float *>(dout),
                                                         lse, delta, static_cast<float *>(dqkv), sg.d_tiles,
                                                         sg.d_tile_of_tok, sg.n_h, heads, D, dh, sg.max_n_tok);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  attn_bwd_f32_kernel<true><<<grid, dim3(128), lds, st>>>(static_cast<const float *>(qkv), static_cast<const float *>(dout),
                                                        lse, delta, static_cast<float *>(dqkv), sg.d_tiles,
                                                        sg.d_tile_of_tok, sg.n_h, heads, D, dh, sg.max_n_tok);
  return hipGetLastError();
}

}  // namespace reslim
