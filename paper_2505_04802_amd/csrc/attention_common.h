// Pieces shared by the tile-attention kernels (forward and gradient): vector types,
// the argument block, the XCD-aware numbering of work units, the fragment row
// permutation, direct-to-LDS loads and hand-issued transposing LDS reads.
#pragma once

#include "common.h"

namespace reslim {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

struct AttnArgs {
  const void *qkv;
  void *out;
  const tile_desc *tiles;
  int T, heads, D, QB, total;
  int64_t n_h;
  float scale_log2;   // log2(e) / sqrt(dh)
  float *lse;         // optional [batch, heads, n_h]: natural log of each query's softmax denominator
  // Stitched output (bf16 kernel only): with Wp > 0 a query that its tile owns writes row
  // b * N + y * Wp + x of `out` (its patch), halo queries write nothing, and units or waves
  // without an owned query do no arithmetic.  Wp == 0: tile-major rows as usual.
  int Wp;
  int64_t N;
};

__device__ __forceinline__ int xcd_remap_attn(int pid, int total) {
  constexpr int NXCD = 8;
  const int x = pid % NXCD, local = pid / NXCD;
  const int q = total / NXCD, r = total % NXCD;
  return x * q + (x < r ? x : r) + local;
}

// A-operand row i of the S^T MFMA carries key perm(i) of the 32-key group:
// swapping bits 2 and 3 makes accumulator registers 8a..8a+7 of lane half `hi`
// hold the 8 consecutive keys 16a + 8hi + (0..7).
__device__ __forceinline__ int key_perm(int i) {
  return (i & 0x13) | ((i & 4) << 1) | ((i & 8) >> 1);
}

typedef __attribute__((ext_vector_type(4))) short s16x4;

// 64 lanes x 16 bytes from global memory to 1 KiB of LDS starting at lds_wave_base
__device__ __forceinline__ void attn_dl_load16(const bf16_t *gsrc, unsigned char *lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)gsrc,
                                   (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

// The V^T fragments of one 32-key group at dh = 64: eight transposing reads issued by
// hand.  As a compiler builtin the read is preceded by a wait for ALL outstanding
// vector-memory operations (the compiler cannot tell that the direct-to-LDS loads in
// flight fill the other stage), which would stall every key block until the next
// block's prefetch has landed.  The reads are issued in one statement and waited for
// in a second one, so independent work can be scheduled in between; LDS operations
// complete in order, so the compiler's own LDS waits stay sufficient.
struct VFrag64 { uint64_t r[2][2][2]; };      // [16-key half][feature block d][e]

template <int OFF>
__device__ __forceinline__ void v_frag_issue(VFrag64 &f, const unsigned (&a)[2][2]) {
  asm volatile(
      "ds_read_b64_tr_b16 %0, %8 offset:%12\n\t"
      "ds_read_b64_tr_b16 %1, %9 offset:%12\n\t"
      "ds_read_b64_tr_b16 %2, %10 offset:%12\n\t"
      "ds_read_b64_tr_b16 %3, %11 offset:%12\n\t"
      "ds_read_b64_tr_b16 %4, %8 offset:%13\n\t"
      "ds_read_b64_tr_b16 %5, %9 offset:%13\n\t"
      "ds_read_b64_tr_b16 %6, %10 offset:%13\n\t"
      "ds_read_b64_tr_b16 %7, %11 offset:%13"
      : "=&v"(f.r[0][0][0]), "=&v"(f.r[0][0][1]), "=&v"(f.r[0][1][0]), "=&v"(f.r[0][1][1]),
        "=&v"(f.r[1][0][0]), "=&v"(f.r[1][0][1]), "=&v"(f.r[1][1][0]), "=&v"(f.r[1][1][1])
      : "v"(a[0][0]), "v"(a[1][0]), "v"(a[0][1]), "v"(a[1][1]), "n"(OFF), "n"(OFF + 16 * 128));
}

__device__ __forceinline__ void v_frag_wait(VFrag64 &f) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(f.r[0][0][0]), "+v"(f.r[0][0][1]), "+v"(f.r[0][1][0]), "+v"(f.r[0][1][1]),
                 "+v"(f.r[1][0][0]), "+v"(f.r[1][0][1]), "+v"(f.r[1][1][0]), "+v"(f.r[1][1][1]));
}

// Exchange between lanes l and l + 32: both get (value of lane l, value of lane l + 32).
// v_permlane32_swap swaps the upper half of its first register with the lower half of its
// second; given two copies of v that leaves the lower lanes' values in both halves of the first
// and the upper lanes' values in both halves of the second.  Inline assembly, because the
// compiler builtin for this instruction hands back its first result for both (checked on the
// device: the sum of the two results came out as twice the first); the waits before and after
// are the ones the compiler places around the instruction itself.
__device__ __forceinline__ void lane_pair_exchange(unsigned v, unsigned &from_lower, unsigned &from_upper) {
  from_lower = v;
  from_upper = v;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(from_lower), "+v"(from_upper));
}

}  // namespace reslim
