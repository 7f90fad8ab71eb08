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
  int64_t n_h;
  int64_t aux_stride;    // records per array
  float c;               // log2(e) / sqrt(dh)
  float sc;              // 1 / sqrt(dh)
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
                                                                 int D, float sqrt_dh, int64_t aux_stride) {
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
    aux[rec] = split3_bf16(-lse[rec] * sqrt_dh);
    aux[aux_stride + rec] = split3_bf16(-acc);
  }
}

template <int OFF>
__device__ __forceinline__ uint64_t tr_issue(unsigned addr) {
  uint64_t r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
  return r;
}

template <int DH, int BS, bool KV, int MINW>
__global__ __launch_bounds__(256, MINW) void attn_bwd_bf16_kernel(AttnBwdArgs a) {
  constexpr int BX = 128;                 // stationary tokens per unit
  constexpr int ROWB = DH * 2;
  constexpr int CPR = DH / 8;
  constexpr int RPB = 64 / CPR;
  constexpr int TILE_B = BS * ROWB;
  constexpr int AUXB = KV ? 2 * BS * 16 : 0;
  constexpr int AUXL = AUXB / 1024;       // wave-loads of the record block
  constexpr int STAGE = 2 * TILE_B + AUXB;
  constexpr int LPW = TILE_B / 1024 / 4;
  constexpr int NKT = BS / 32, NKS = DH / 16, NDT = DH / 32;
  constexpr bool HAND = DH == 64;         // transposing reads issued by hand (see attention_common.h)
  static_assert(TILE_B % 4096 == 0 && AUXB % 1024 == 0 && 2 * STAGE <= 160 * 1024, "LDS plan");
  extern __shared__ __align__(1024) unsigned char smem[];   // 2 * STAGE bytes (above 64 KiB at dh = 256)

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

  struct Unit {
    int n_t, r0, nsb;
    const bf16_t *x1, *x2, *y1, *y2;
    const u32x4 *aux;     // record 0 of this (sample, head, tile) in array 0
    bf16_t *o1, *o2;
  };
  auto decode = [&](int vb, Unit &u) -> int {
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
        const size_t row0 = static_cast<size_t>(b) * a.n_h + a.tiles[tile].tok_off;
        const bf16_t *q = a.qkv + row0 * ldq + head * DH;
        const bf16_t *d_o = a.dout + row0 * a.D + head * DH;
        bf16_t *dq = a.dqkv + row0 * ldq + head * DH;
        u.n_t = n_t;
        u.r0 = xb * BX;
        u.nsb = (n_t + BS - 1) / BS;
        u.x1 = KV ? q + a.D : q;
        u.x2 = KV ? q + 2 * a.D : d_o;
        u.y1 = KV ? q : q + a.D;
        u.y2 = KV ? d_o : q + 2 * a.D;
        u.aux = a.aux + (static_cast<size_t>(b) * a.heads + head) * a.n_h + a.tiles[tile].tok_off;
        u.o1 = KV ? dq + a.D : dq;
        u.o2 = dq + 2 * a.D;
        return vb;
      }
      vb += G;
    }
    return vb;
  };
  Unit cur, nxt;
  int vb = decode(blockIdx.x, cur);
  if (vb >= a.total) return;
  vb = decode(vb + G, nxt);
  bool has_next = vb < a.total;

  // ---- load side
  int ld_row[LPW], off1[LPW], off2[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    ld_row[i] = (wave + 4 * i) * RPB + lane / CPR;
    const int ch = ((lane % CPR) ^ swz(ld_row[i])) * 16;
    off1[i] = ld_row[i] * ldq * 2 + ch;
    off2[i] = ld_row[i] * ldy2 * 2 + ch;
  }
  const int aux_L = wave * 64 + lane;                 // record slot of this lane in the block (KV only)
  const int aux_arr = aux_L / BS, aux_row = aux_L % BS;
  auto issue = [&](const Unit &u, int s0, int buf) {
    unsigned char *sb = smem + buf * STAGE;
    const unsigned char *g1 = reinterpret_cast<const unsigned char *>(u.y1 + static_cast<size_t>(s0) * ldq);
    const unsigned char *g2 = reinterpret_cast<const unsigned char *>(u.y2 + static_cast<size_t>(s0) * ldy2);
    const int lim = u.n_t - 1 - s0;       // last valid row of this block
    if (lim >= BS - 1) {
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        attn_dl_load16(reinterpret_cast<const bf16_t *>(g1 + static_cast<uint32_t>(off1[i])), sb + (wave + 4 * i) * 1024);
        attn_dl_load16(reinterpret_cast<const bf16_t *>(g2 + static_cast<uint32_t>(off2[i])),
                       sb + TILE_B + (wave + 4 * i) * 1024);
      }
    } else {                               // rows past the tile end re-read its last row (finite; masked later)
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        const int back = max(ld_row[i] - lim, 0);
        attn_dl_load16(reinterpret_cast<const bf16_t *>(g1 + static_cast<uint32_t>(off1[i] - back * ldq * 2)),
                       sb + (wave + 4 * i) * 1024);
        attn_dl_load16(reinterpret_cast<const bf16_t *>(g2 + static_cast<uint32_t>(off2[i] - back * ldy2 * 2)),
                       sb + TILE_B + (wave + 4 * i) * 1024);
      }
    }
    if constexpr (KV) {
      if (wave < AUXL) {
        const int row = s0 + min(aux_row, lim);
        attn_dl_load16(reinterpret_cast<const bf16_t *>(u.aux + aux_arr * a.aux_stride + row), sb + 2 * TILE_B + wave * 1024);
      }
    }
  };
  bf16x8 x1f[NKS], x2f[NKS];
  f32x16 sinit, dpinit;
  auto load_x = [&](const Unit &u) {
    const int xrow = min(u.r0 + wave * 32 + l32, u.n_t - 1);
    const bf16_t *p1 = u.x1 + static_cast<size_t>(xrow) * ldq + hi * 8;
    const bf16_t *p2 = u.x2 + static_cast<size_t>(xrow) * ldx2 + hi * 8;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      x1f[ks] = *reinterpret_cast<const bf16x8 *>(p1 + ks * 16);
      x2f[ks] = *reinterpret_cast<const bf16x8 *>(p2 + ks * 16);
    }
    float si = 0.f, di = 0.f;
    if constexpr (!KV) {
      const u32x2 r0 = *reinterpret_cast<const u32x2 *>(u.aux + xrow);
      const u32x2 r1 = *reinterpret_cast<const u32x2 *>(u.aux + a.aux_stride + xrow);
      si = join3_bf16(r0[0], r0[1]);
      di = join3_bf16(r1[0], r1[1]);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) { sinit[r] = si; dpinit[r] = di; }
  };

  // ---- read side
  const int yr = key_perm(l32);
  const int y_row = yr * ROWB, y_swz = swz(yr);
  const int L16 = lane & 15;
  int t_addr[2][NDT];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int vr = 8 * hi + 4 * e + (L16 >> 2);
#pragma unroll
    for (int d = 0; d < NDT; ++d) {
      const int o = 32 * d + 16 * ((lane >> 4) & 1) + 4 * (L16 & 3);
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

  f32x16 acc1[NDT], acc2[KV ? NDT : 1];
  auto reset = [&]() {
#pragma unroll
    for (int d = 0; d < NDT; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc1[d][r] = 0.f;
#pragma unroll
    for (int d = 0; d < (KV ? NDT : 1); ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc2[d][r] = 0.f;
  };
  reset();
  load_x(cur);
  issue(cur, 0, 0);

  int sb = 0;
  for (int g = 0;; ++g) {
    __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0)
    __syncthreads();
    const bool last = sb + 1 == cur.nsb;
    if (!last) issue(cur, (sb + 1) * BS, (g + 1) & 1);
    else if (has_next) issue(nxt, 0, (g + 1) & 1);
    const unsigned char *st = smem + (g & 1) * STAGE;
    const int s0 = sb * BS;
    const bool active = cur.r0 + wave * 32 < cur.n_t;

    // one 32-token group of the streamed block at a time: scores, probabilities, then the
    // two products that consume them (keeps one pair of score accumulators live)
    auto group = [&](auto kt_c, bool fetch_next) {
      constexpr int kt = decltype(kt_c)::value;
      f32x16 s, dp;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const unsigned char *rp = st + kt * 32 * ROWB + y_row + (((2 * ks + hi) ^ y_swz) << 4);
        const bf16x8 f1 = *reinterpret_cast<const bf16x8 *>(rp);
        const bf16x8 f2 = *reinterpret_cast<const bf16x8 *>(rp + TILE_B);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1, x1f[ks], ks == 0 ? sinit : s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f2, x2f[ks], ks == 0 ? dpinit : dp, 0, 0, 0);
      }
      if constexpr (KV) {
        const bf16x8 fa = *reinterpret_cast<const bf16x8 *>(st + aux_addr + kt * 32 * 16);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, ones_s, s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, ones_d, dp, 0, 0, 0);
      }
      // the stationary fragments are dead after the last scores of a unit: fetch the next unit's
      if (fetch_next) load_x(nxt);
      if (s0 + kt * 32 + 32 > cur.n_t) {   // ragged end: streamed tokens past the tile end get probability 0
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = s0 + kt * 32 + 16 * (r / 8) + 8 * hi + (r % 8);
          if (row >= cur.n_t) s[r] = -INFINITY;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[r] = __builtin_amdgcn_exp2f(s[r] * a.c);
        dp[r] *= s[r];
      }
      const unsigned st_off = static_cast<unsigned>(reinterpret_cast<uintptr_t>(
          (__attribute__((address_space(3))) const unsigned char *)st));
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
              r1[d][e] = tr_issue<ROFF>(st_off + static_cast<unsigned>(t_addr[e][d]));
              if constexpr (KV) r2[d][e] = tr_issue<ROFF + TILE_B>(st_off + static_cast<unsigned>(t_addr[e][d]));
            }
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            dsf[e] = static_cast<__bf16>(dp[8 * h2 + e]);
            if constexpr (KV) pf[e] = static_cast<__bf16>(s[8 * h2 + e]);
          }
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
          for (int d = 0; d < NDT; ++d)
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              asm volatile("" : "+v"(r1[d][e]));
              if constexpr (KV) asm volatile("" : "+v"(r2[d][e]));
            }
#pragma unroll
          for (int d = 0; d < NDT; ++d) {
            const u64x2 b1 = {r1[d][0], r1[d][1]};
            acc1[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b1), dsf, acc1[d], 0, 0, 0);
            if constexpr (KV) {
              const u64x2 b2 = {r2[d][0], r2[d][1]};
              acc2[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b2), pf, acc2[d], 0, 0, 0);
            }
          }
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            dsf[e] = static_cast<__bf16>(dp[8 * h2 + e]);
            if constexpr (KV) pf[e] = static_cast<__bf16>(s[8 * h2 + e]);
          }
          typedef __attribute__((ext_vector_type(8))) short s16x8;
#pragma unroll
          for (int d = 0; d < NDT; ++d) {
            const unsigned char *vp = st + ROFF;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3))) *)(vp + t_addr[0][d]));
            const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (s16x4 __attribute__((address_space(3))) *)(vp + t_addr[1][d]));
            const s16x8 both = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
            acc1[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both), dsf, acc1[d], 0, 0, 0);
            if constexpr (KV) {
              const s16x4 lo2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                  (s16x4 __attribute__((address_space(3))) *)(vp + TILE_B + t_addr[0][d]));
              const s16x4 hi2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                  (s16x4 __attribute__((address_space(3))) *)(vp + TILE_B + t_addr[1][d]));
              const s16x8 both2 = __builtin_shufflevector(lo2, hi2, 0, 1, 2, 3, 4, 5, 6, 7);
              acc2[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, both2), pf, acc2[d], 0, 0, 0);
            }
          }
        }
      };
      step(std::integral_constant<int, 0>{});
      step(std::integral_constant<int, 1>{});
    };
    static_assert(NKT <= 2, "streamed block of 32 or 64 tokens");
    const bool fetch = last && has_next;
    if (active) {
      const bool two = NKT == 2 && s0 + 32 < cur.n_t;      // the second group holds at least one token
      group(std::integral_constant<int, 0>{}, fetch && !two);
      if constexpr (NKT == 2) {
        if (two) group(std::integral_constant<int, 1>{}, fetch);
      }
    } else if (fetch) {
      load_x(nxt);
    }
    if (!last) { ++sb; continue; }

    // ---- end of a unit: scale, round and store this lane's row of each gradient
    const int xrow = cur.r0 + wave * 32 + l32;
    if (active && xrow < cur.n_t) {
      bf16_t *p1 = cur.o1 + static_cast<size_t>(xrow) * ldq + hi * 4;
      bf16_t *p2 = cur.o2 + static_cast<size_t>(xrow) * ldq + hi * 4;
#pragma unroll
      for (int d = 0; d < NDT; ++d)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          bf16x4 tmp;
#pragma unroll
          for (int e = 0; e < 4; ++e) tmp[e] = static_cast<__bf16>(acc1[d][4 * r4 + e] * a.sc);
          *reinterpret_cast<u32x2 *>(p1 + d * 32 + r4 * 8) = __builtin_bit_cast(u32x2, tmp);
          if constexpr (KV) {
#pragma unroll
            for (int e = 0; e < 4; ++e) tmp[e] = static_cast<__bf16>(acc2[d][4 * r4 + e]);
            *reinterpret_cast<u32x2 *>(p2 + d * 32 + r4 * 8) = __builtin_bit_cast(u32x2, tmp);
          }
        }
    }
    if (!has_next) break;
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

template <int DH, int BS>
constexpr int bwd_lds_bytes(bool kv) { return 2 * (2 * BS * DH * 2 + (kv ? 2 * BS * 16 : 0)); }

static int g_bwd_cus = 0;
static bool g_bwd_dh256_ok = false;

hipError_t attention_bwd_init() {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&g_bwd_cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  // the key-stationary kernel at dh = 256 needs 66 KiB of LDS, above the default limit of a launch
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bwd_bf16_kernel<256, 32, true, 1>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, bwd_lds_bytes<256, 32>(true));
  g_bwd_dh256_ok = e == hipSuccess;
  if (e != hipSuccess) (void)hipGetLastError();    // not fatal: only the dh = 256 gradient is refused
  return hipSuccess;
}

size_t tiles_attention_bwd_ws_bytes(const reslim_ctx *c, int batch) {
  const size_t recs = static_cast<size_t>(batch) * c->cfg.heads * c->n_h;
  return c->cfg.dtype == RESLIM_BF16 ? align256(recs * 32) : align256(recs * 4);
}

template <int DH, int BS, int MINW_Q, int MINW_KV>
static hipError_t launch_bwd_pair(const AttnBwdArgs &a, hipStream_t st) {
  const int gq = a.total < MINW_Q * g_bwd_cus ? a.total : MINW_Q * g_bwd_cus;
  const int gk = a.total < MINW_KV * g_bwd_cus ? a.total : MINW_KV * g_bwd_cus;
  attn_bwd_bf16_kernel<DH, BS, false, MINW_Q><<<dim3(gq), dim3(256), bwd_lds_bytes<DH, BS>(false), st>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  attn_bwd_bf16_kernel<DH, BS, true, MINW_KV><<<dim3(gk), dim3(256), bwd_lds_bytes<DH, BS>(true), st>>>(a);
  return hipGetLastError();
}

hipError_t launch_tiles_attention_bwd(const reslim_ctx *c, const void *qkv, const void *out, const float *lse,
                                      const void *dout, void *dqkv, int batch, void *ws, hipStream_t st) {
  const int heads = c->cfg.heads, D = c->cfg.embed_dim, dh = c->dh;
  const int64_t recs = static_cast<int64_t>(batch) * heads * c->n_h;
  if (recs == 0) return hipSuccess;
  if (c->cfg.dtype == RESLIM_BF16) {
    AttnBwdArgs a;
    a.qkv = static_cast<const bf16_t *>(qkv);
    a.dout = static_cast<const bf16_t *>(dout);
    a.aux = static_cast<const u32x4 *>(ws);
    a.dqkv = static_cast<bf16_t *>(dqkv);
    a.tiles = c->d_tiles;
    a.T = c->T;
    a.heads = heads;
    a.D = D;
    a.n_h = c->n_h;
    a.aux_stride = recs;
    a.c = 1.4426950408889634f / sqrtf(static_cast<float>(dh));
    a.sc = 1.0f / sqrtf(static_cast<float>(dh));
    a.QB = (c->max_n_tok + 127) / 128;
    const int64_t total = static_cast<int64_t>(batch) * c->T * heads * a.QB;
    if (total > INT32_MAX || g_bwd_cus <= 0) return hipErrorInvalidValue;
    a.total = static_cast<int>(total);
    const int64_t n_vec = static_cast<int64_t>(batch) * c->n_h * D / 8;
    const unsigned pg = static_cast<unsigned>((n_vec + 255) / 256);
    const float sq = sqrtf(static_cast<float>(dh));
    u32x4 *aux = static_cast<u32x4 *>(ws);
    const bf16_t *o = static_cast<const bf16_t *>(out);
    switch (dh) {
      case 64: attn_bwd_prep_bf16_kernel<64><<<dim3(pg), dim3(256), 0, st>>>(o, a.dout, lse, aux, n_vec, c->n_h, heads, D, sq, recs); break;
      case 128: attn_bwd_prep_bf16_kernel<128><<<dim3(pg), dim3(256), 0, st>>>(o, a.dout, lse, aux, n_vec, c->n_h, heads, D, sq, recs); break;
      case 256: attn_bwd_prep_bf16_kernel<256><<<dim3(pg), dim3(256), 0, st>>>(o, a.dout, lse, aux, n_vec, c->n_h, heads, D, sq, recs); break;
      default: return hipErrorInvalidValue;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    switch (dh) {
      case 64: return launch_bwd_pair<64, 64, 2, 2>(a, st);
      case 128: return launch_bwd_pair<128, 32, 2, 1>(a, st);
      default: return g_bwd_dh256_ok ? launch_bwd_pair<256, 32, 1, 1>(a, st) : hipErrorInvalidValue;
    }
  }
  float *delta = static_cast<float *>(ws);
  const size_t lds = (2 * static_cast<size_t>(c->max_n_tok) + 2 * dh) * sizeof(float);
  if (lds > 60 * 1024 || c->n_h > INT32_MAX) return hipErrorInvalidValue;
  const int64_t n = static_cast<int64_t>(batch) * c->n_h * heads;
  attn_bwd_delta_f32_kernel<<<dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st>>>(
      static_cast<const float *>(out), static_cast<const float *>(dout), delta, n, c->n_h, heads, dh);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid(static_cast<unsigned>(c->n_h), heads, batch);
  attn_bwd_f32_kernel<false><<<grid, dim3(128), lds, st>>>(static_cast<const float *>(qkv), static_cast<const float *>(dout),
                                                         lse, delta, static_cast<float *>(dqkv), c->d_tiles,
                                                         c->d_tile_of_tok, c->n_h, heads, D, dh, c->max_n_tok);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  attn_bwd_f32_kernel<true><<<grid, dim3(128), lds, st>>>(static_cast<const float *>(qkv), static_cast<const float *>(dout),
                                                        lse, delta, static_cast<float *>(dqkv), c->d_tiles,
                                                        c->d_tile_of_tok, c->n_h, heads, D, dh, c->max_n_tok);
  return hipGetLastError();
}

}  // namespace reslim
