// Weight gradient of a linear layer y = x W^T + b (training of the model of ORBIT-2
// Sec. 4.1; the chain rule gives  dW[n][k] = sum_m dY[m][n] * X[m][k]):  a contraction over
// the TOKENS, the leading index of both operands, so neither is "k-contiguous" the way the
// forward GEMM wants them.  Instead of transposing activations in HBM the kernel reads both
// operands as they lie, [token][feature] row-major:
//   * token blocks of BM rows go global -> LDS directly (global_load_lds_dwordx4), two stages,
//     rows XOR-swizzled in 16-byte chunks;
//   * both MFMA operands are fetched with the TRANSPOSING LDS read ds_read_b64_tr_b16: a lane
//     gets 8 consecutive tokens of one feature column, which is exactly the k-slice of an
//     A operand (feature = output row n, from dY) or a B operand (feature = k, from X);
//   * a work-group owns a TN x TK tile of dW for a slice of the tokens (split over tokens:
//     dW is small and M is huge); fp32 partial tiles are summed in a fixed order afterwards
//     (deterministic, no atomics).
#include <type_traits>

#include "attention_common.h"

namespace reslim {

struct WgradArgs {
  const bf16_t *dy;      // [M, N]
  const bf16_t *x;       // [M, K]
  float *out;            // [S, N, K] partial tiles (S = 1: the gradient itself)
  const void *zeros;     // >= 16 readable zero bytes, 16-byte aligned
  int M, N, K;
  int m_per_split;       // tokens per split, a multiple of BM
  int tiles_k;           // tiles along K
};

template <int TN, int TK, int NWAVE, int BM, int MINW>
__global__ __launch_bounds__(64 * NWAVE, MINW) void wgrad_bf16_kernel(WgradArgs a) {
  constexpr int WR = TN / 64, WC = NWAVE / WR;      // waves along n and along k; a wave owns 64 x WKW
  constexpr int WKW = TK / WC, NBK = WKW / 32;
  constexpr int ROWN = TN * 2, ROWK = TK * 2;       // bytes per LDS row of the two tiles
  constexpr int CPRN = TN / 8, CPRK = TK / 8;       // 16-byte chunks per row
  constexpr int TILE_N = BM * ROWN, TILE_K = BM * ROWK, STAGE = TILE_N + TILE_K;
  constexpr int LN = TILE_N / 1024 / NWAVE, LK = TILE_K / 1024 / NWAVE;   // wave-loads per wave and operand
  static_assert(WR * WC == NWAVE && WKW % 32 == 0 && TILE_N % (1024 * NWAVE) == 0 && TILE_K % (1024 * NWAVE) == 0, "tiling");
  static_assert(CPRN >= 16 && CPRK >= 16 && 2 * STAGE <= 65536 && BM % 16 == 0, "LDS plan");
  __shared__ __align__(1024) unsigned char smem[2 * STAGE];

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int hi = lane >> 5, l32 = lane & 31, L16 = lane & 15;
  const int wn = wave / WC, wk = wave % WC;
  const int tile = blockIdx.x;
  const int n0 = (tile / a.tiles_k) * TN, k0 = (tile % a.tiles_k) * TK;
  const int m_begin = blockIdx.y * a.m_per_split;
  const int m_end = min(a.M, m_begin + a.m_per_split);
  const int nblk = (m_end - m_begin + BM - 1) / BM;
  // rows 4r .. 4r+3 hit the same banks unless their chunks are moved apart: chunk ^= swz(row)
  auto swz = [](int r) { return ((r & 3) << 2) | ((r >> 2) & 3); };

  // ---- load side: lane -> (row of the block, chunk) for each of its wave-loads
  auto issue = [&](int blk, int buf) {
    unsigned char *sb = smem + buf * STAGE;
    const int m0 = m_begin + blk * BM;
#pragma unroll
    for (int i = 0; i < LN; ++i) {
      const int wl = wave + NWAVE * i;
      const int row = wl * (64 / CPRN) + lane / CPRN;
      const int ch = (lane % CPRN) ^ swz(row);
      const bool ok = m0 + row < m_end && n0 + ch * 8 < a.N;
      const bf16_t *src = ok ? a.dy + static_cast<size_t>(m0 + row) * a.N + n0 + ch * 8 : static_cast<const bf16_t *>(a.zeros);
      attn_dl_load16(src, sb + wl * 1024);
    }
#pragma unroll
    for (int i = 0; i < LK; ++i) {
      const int wl = wave + NWAVE * i;
      const int row = wl * (64 / CPRK) + lane / CPRK;
      const int ch = (lane % CPRK) ^ swz(row);
      const bool ok = m0 + row < m_end && k0 + ch * 8 < a.K;
      const bf16_t *src = ok ? a.x + static_cast<size_t>(m0 + row) * a.K + k0 + ch * 8 : static_cast<const bf16_t *>(a.zeros);
      attn_dl_load16(src, sb + TILE_N + wl * 1024);
    }
  };

  // ---- read side: this lane points at token row 8*hi + 4*e + (lane%16)/4 of a 16-token step
  // and at the 4 features 32*d + 16*((lane/16)&1) + 4*(lane%4) .. +3 of feature block d
  unsigned ta[2][2], tb[2][NBK];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int vr = 8 * hi + 4 * e + (L16 >> 2);
    const int fo = 16 * ((lane >> 4) & 1) + 4 * (L16 & 3);
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int o = 32 * (wn * 2 + nb) + fo;
      ta[e][nb] = vr * ROWN + (((o >> 3) ^ swz(vr)) << 4) + ((o >> 2) & 1) * 8;
    }
#pragma unroll
    for (int kb = 0; kb < NBK; ++kb) {
      const int o = 32 * (wk * NBK + kb) + fo;
      tb[e][kb] = TILE_N + vr * ROWK + (((o >> 3) ^ swz(vr)) << 4) + ((o >> 2) & 1) * 8;
    }
  }

  f32x16 acc[2][NBK];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int kb = 0; kb < NBK; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[nb][kb][r] = 0.f;

  const bool live = n0 + wn * 64 < a.N && k0 + wk * WKW < a.K;     // this wave's sub-tile holds outputs
  if (nblk > 0) issue(0, 0);
  for (int g = 0; g < nblk; ++g) {
    __builtin_amdgcn_s_waitcnt(0x0F70);       // vmcnt(0): this wave's part of block g is in LDS
    __builtin_amdgcn_s_barrier();             // ... and everybody's; the other stage is free
    if (g + 1 < nblk) issue(g + 1, (g + 1) & 1);
    if (!live) continue;
    const unsigned st_off = static_cast<unsigned>(reinterpret_cast<uintptr_t>(
        (__attribute__((address_space(3))) const unsigned char *)(smem + (g & 1) * STAGE)));
    auto step = [&](auto ms_c) {
      constexpr int ms = decltype(ms_c)::value;
      uint64_t fa[2][2], fb[NBK][2];
      // the transposing reads are issued by hand: as compiler builtins each would be preceded by
      // a wait for all vector-memory operations, i.e. for the prefetch just issued
#pragma unroll
      for (int e = 0; e < 2; ++e) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(fa[nb][e]) : "v"(st_off + ta[e][nb]), "n"(ms * 16 * ROWN));
        }
#pragma unroll
        for (int kb = 0; kb < NBK; ++kb) {
          asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(fb[kb][e]) : "v"(st_off + tb[e][kb]), "n"(ms * 16 * ROWK));
        }
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int e = 0; e < 2; ++e) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) asm volatile("" : "+v"(fa[nb][e]));
#pragma unroll
        for (int kb = 0; kb < NBK; ++kb) asm volatile("" : "+v"(fb[kb][e]));
      }
      typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const u64x2 av = {fa[nb][0], fa[nb][1]};
#pragma unroll
        for (int kb = 0; kb < NBK; ++kb) {
          const u64x2 bv = {fb[kb][0], fb[kb][1]};
          acc[nb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, bv),
                                                                 acc[nb][kb], 0, 0, 0);
        }
      }
    };
    step(std::integral_constant<int, 0>{});
    step(std::integral_constant<int, 1>{});
    if constexpr (BM == 64) {
      step(std::integral_constant<int, 2>{});
      step(std::integral_constant<int, 3>{});
    }
    static_assert(BM == 32 || BM == 64, "two or four 16-token steps per block");
  }

  // ---- store: accumulator register r of lane (l32, hi) is row 8*(r/4) + 4*hi + r%4, column l32
  if (!live) return;
  float *out = a.out + static_cast<size_t>(blockIdx.y) * a.N * a.K;
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int kb = 0; kb < NBK; ++kb) {
      const int k = k0 + (wk * NBK + kb) * 32 + l32;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int n = n0 + (wn * 2 + nb) * 32 + 8 * (r / 4) + 4 * hi + (r % 4);
        if (n < a.N && k < a.K) out[static_cast<size_t>(n) * a.K + k] = acc[nb][kb][r];
      }
    }
}

// fp32 debug path: one thread per element of dW
__global__ __launch_bounds__(256) void wgrad_f32_kernel(const float *__restrict__ dy, const float *__restrict__ x,
                                                        float *__restrict__ out, int M, int N, int K) {
  const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx >= static_cast<int64_t>(N) * K) return;
  const int n = static_cast<int>(idx / K), k = static_cast<int>(idx % K);
  float acc = 0.f;
  for (int m = 0; m < M; ++m) acc = fmaf(dy[static_cast<size_t>(m) * N + n], x[static_cast<size_t>(m) * K + k], acc);
  out[idx] = acc;
}

static int g_wgrad_cus = 0;
hipError_t wgrad_init() {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  return hipDeviceGetAttribute(&g_wgrad_cus, hipDeviceAttributeMultiprocessorCount, dev);
}

struct WgradPlan { bool big; int tiles_n, tiles_k, splits, m_per_split; };
static WgradPlan wgrad_plan(int M, int N, int K) {
  WgradPlan p;
  p.big = N % 256 == 0 && K % 256 == 0;
  const int tn = p.big ? 256 : 128;
  p.tiles_n = (N + tn - 1) / tn;
  p.tiles_k = (K + tn - 1) / tn;
  const int tiles = p.tiles_n * p.tiles_k;
  const int cus = g_wgrad_cus > 0 ? g_wgrad_cus : 256;
  // splits so that tiles * splits fills ONE round of resident work-groups without spilling into a
  // second, nearly empty one (the 8-wave kernel holds one work-group per CU, the 4-wave one four)
  const int slots = p.big ? cus : 4 * cus;
  int s = slots / tiles;
  const int max_s = (M + 255) / 256;                  // at least 256 tokens per split
  s = s < 1 ? 1 : (s > max_s ? max_s : s);
  if (s > 64) s = 64;
  int mps = (M + s - 1) / s;
  mps = (mps + 31) / 32 * 32;
  p.splits = (M + mps - 1) / mps;
  p.m_per_split = mps;
  return p;
}

// bytes of fp32 scratch the weight gradient of an [M, N] x [M, K] pair needs (0: none)
size_t wgrad_ws_bytes(int dtype, int M, int N, int K) {
  if (dtype != RESLIM_BF16) return 0;
  const WgradPlan p = wgrad_plan(M, N, K);
  return p.splits > 1 ? align256(static_cast<size_t>(p.splits) * N * K * sizeof(float)) : 0;
}

hipError_t launch_partial_reduce(const float *partial, float *out, int n_part, int64_t stride, int64_t n, hipStream_t st);

// dW[N, K] (fp32) = dY[M, N]^T X[M, K]; ws as sized by wgrad_ws_bytes
hipError_t launch_wgrad(int dtype, const void *dy, const void *x, float *dw, int M, int N, int K, void *ws,
                        const void *zeros, hipStream_t st) {
  if (M <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;
  if (dtype != RESLIM_BF16) {
    const int64_t n = static_cast<int64_t>(N) * K;
    wgrad_f32_kernel<<<dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st>>>(
        static_cast<const float *>(dy), static_cast<const float *>(x), dw, M, N, K);
    return hipGetLastError();
  }
  if (N % 8 != 0 || K % 8 != 0) return hipErrorInvalidValue;
  const WgradPlan p = wgrad_plan(M, N, K);
  WgradArgs a;
  a.dy = static_cast<const bf16_t *>(dy);
  a.x = static_cast<const bf16_t *>(x);
  a.out = p.splits > 1 ? static_cast<float *>(ws) : dw;
  a.zeros = zeros;
  a.M = M;
  a.N = N;
  a.K = K;
  a.m_per_split = p.m_per_split;
  a.tiles_k = p.tiles_k;
  if (p.splits > 1 && !ws) return hipErrorInvalidValue;
  const dim3 grid(p.tiles_n * p.tiles_k, p.splits);
  if (p.big) wgrad_bf16_kernel<256, 256, 8, 32, 1><<<grid, dim3(512), 0, st>>>(a);
  else wgrad_bf16_kernel<128, 128, 4, 32, 2><<<grid, dim3(256), 0, st>>>(a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.splits == 1) return e;
  return launch_partial_reduce(static_cast<const float *>(ws), dw, p.splits, static_cast<int64_t>(N) * K,
                               static_cast<int64_t>(N) * K, st);
}

}  // namespace reslim
