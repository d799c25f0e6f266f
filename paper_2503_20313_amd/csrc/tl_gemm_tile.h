// One bf16 GEMM output tile on CDNA4 matrix cores: C[BM,BN] = A[BM,K] . B[K,BN], A row-major
// (K contiguous), B row-major as [K,N] (N contiguous), fp32 accumulation, bf16 (RNE) output.
//
// Design (gfx950):
//  * global -> LDS with 16-byte direct-to-LDS loads (no register staging), two stages; the
//    bijection between 16-byte chunks and LDS slots is chosen so that the later fragment reads
//    are bank-conflict free (A: chunk index XOR (row/2)%8; B with a power-of-two row pitch:
//    64-byte group XOR k%4; B tiles 224 wide need none).
//  * the MFMA "A" operand is taken from the B tile with transposing LDS reads
//    (ds_read_b64_tr_b16: a 16-lane block reads 4 k-rows x 16 columns and hands each lane the
//    4 k-values of its column), the MFMA "B" operand from the A tile with 16-byte reads; the
//    product is therefore the transposed tile C^T, whose accumulator layout gives every lane
//    4 consecutive columns of one row of C, i.e. 8-byte stores.
//  * v_mfma_f32_32x32x16_bf16, wave tile (BM/WM) x (BN/WN).
#pragma once
#include "tl_device.h"

namespace tl {

template <int BM_, int BN_, int WM_, int WN_>
struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = 64, WM = WM_, WN = WN_;
  static constexpr int NWAVES = WM * WN, NTHREADS = NWAVES * 64;
  static constexpr int WTM = BM / WM, WTN = BN / WN, MT = WTM / 32, NT = WTN / 32;
  static constexpr int A_LOADS = BM * 8 / 64;  // wave-wide 1 KiB loads per stage, A tile
  static constexpr int B_CPR = BN / 8;         // 16-byte chunks per k-row of the B tile
  static constexpr int B_LOADS = B_CPR;        // 64 k-rows * B_CPR chunks / 64 lanes
  static constexpr bool B_SWZ = (B_CPR % 16) == 0;
  static constexpr int A_BYTES = BM * 128, B_BYTES = 64 * BN * 2, STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of the 32x32 MFMA");
};

__device__ __forceinline__ void lds_load16(const void* g, char* lds_wave_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)g,
                                   (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

__device__ __forceinline__ short4_t lds_read_tr(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t*)p);
}

// Computes one output tile.  `a` points at the tile's first row (column 0), `b` at row 0 of B
// at the tile's first column, `c` at the tile's first element.  rows/cols = valid extent of
// the tile (ragged edges): loads are clamped to valid memory, stores are masked.  K % 64 == 0.
// All threads of the workgroup must call it; it ends with all LDS reads complete.
template <class Cfg>
__device__ __forceinline__ void gemm_tile(const bf16_t* __restrict__ a, long lda, const bf16_t* __restrict__ b, long ldb,
                                          bf16_t* __restrict__ c, long ldc, int rows, int cols, int K, char* smem) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / Cfg::WN, wn = wave % Cfg::WN;

  // ---- per-lane global addresses of this wave's share of the stage loads
  constexpr int A_PER_WAVE = (Cfg::A_LOADS + Cfg::NWAVES - 1) / Cfg::NWAVES;
  constexpr int B_PER_WAVE = (Cfg::B_LOADS + Cfg::NWAVES - 1) / Cfg::NWAVES;
  const char* a_src[A_PER_WAVE];
  const char* b_src[B_PER_WAVE];
#pragma unroll
  for (int i = 0; i < A_PER_WAVE; i++) {
    int j = wave + i * Cfg::NWAVES;           // wave-load index: LDS slots [64j, 64j+64)
    int row = j * 8 + (lane >> 3);
    int chunk = (lane & 7) ^ ((row >> 1) & 7);  // logical 16-byte chunk stored at this slot
    int grow = row < rows ? row : rows - 1;
    a_src[i] = (const char*)(a + (long)grow * lda + chunk * 8);
  }
#pragma unroll
  for (int i = 0; i < B_PER_WAVE; i++) {
    int j = wave + i * Cfg::NWAVES;
    int slot = j * 64 + lane;
    int k = slot / Cfg::B_CPR, ncp = slot - k * Cfg::B_CPR;
    int nc = Cfg::B_SWZ ? (ncp ^ ((k & 3) << 2)) : ncp;
    int col = nc * 8 < cols ? nc * 8 : cols - 8;
    b_src[i] = (const char*)(b + (long)k * ldb + col);
  }
  const long b_step = ldb * 64 * 2;  // bytes per K-step

  auto issue_stage = [&](int stage) {
    char* sa = smem + stage * Cfg::STAGE_BYTES;
    char* sb = sa + Cfg::A_BYTES;
#pragma unroll
    for (int i = 0; i < A_PER_WAVE; i++) {
      int j = wave + i * Cfg::NWAVES;
      if (Cfg::A_LOADS % Cfg::NWAVES == 0 || j < Cfg::A_LOADS) lds_load16(a_src[i], sa + j * 1024);
      a_src[i] += 128;
    }
#pragma unroll
    for (int i = 0; i < B_PER_WAVE; i++) {
      int j = wave + i * Cfg::NWAVES;
      if (Cfg::B_LOADS % Cfg::NWAVES == 0 || j < Cfg::B_LOADS) lds_load16(b_src[i], sb + j * 1024);
      b_src[i] += b_step;
    }
  };

  // ---- per-lane LDS read offsets
  // A fragment (MFMA B operand): lane holds row (lane%32) of the wave's m-tile, k = 8*(lane/32)..+7 of the 16-wide k-slice.
  const int a_row = wm * Cfg::WTM + (lane & 31);
  const int a_x = (lane >> 5) ^ ((a_row >> 1) & 7);
  const int a_off = a_row * 128;
  // B fragment (MFMA A operand) via transposing reads: lane supplies the address of k-row
  // 8*(lane/32) + (lane%16)/4 (+4 for the second read), columns 16*((lane/16)%2) + 4*(lane%4)..+3.
  const int b_k = 8 * (lane >> 5) + ((lane & 15) >> 2);
  const int b_n = wn * Cfg::WTN + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  int b_off[Cfg::NT];
#pragma unroll
  for (int nt = 0; nt < Cfg::NT; nt++) {
    int n = b_n + nt * 32;
    int nc = n >> 3;
    if (Cfg::B_SWZ) nc ^= (b_k & 3) << 2;
    b_off[nt] = (b_k * Cfg::B_CPR + nc) * 16 + (n & 4) * 2;
  }

  floatx16 acc[Cfg::MT][Cfg::NT];
#pragma unroll
  for (int mt = 0; mt < Cfg::MT; mt++)
#pragma unroll
    for (int nt = 0; nt < Cfg::NT; nt++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[mt][nt][e] = 0.f;

  const int nk = K / 64;
  issue_stage(0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  for (int kt = 0; kt < nk; kt++) {
    if (kt + 1 < nk) issue_stage((kt + 1) & 1);
    const char* sa = smem + (kt & 1) * Cfg::STAGE_BYTES;
    const char* sb = sa + Cfg::A_BYTES;
#pragma unroll
    for (int kk = 0; kk < 4; kk++) {
      bf16x8 af[Cfg::MT], bfr[Cfg::NT];
#pragma unroll
      for (int mt = 0; mt < Cfg::MT; mt++)
        af[mt] = *(const bf16x8*)(sa + a_off + mt * 32 * 128 + ((a_x ^ (2 * kk)) << 4));
#pragma unroll
      for (int nt = 0; nt < Cfg::NT; nt++) {
        const char* p = sb + b_off[nt] + kk * 16 * Cfg::B_CPR * 16;
        short4_t lo = lds_read_tr(p);
        short4_t hi = lds_read_tr(p + 4 * Cfg::B_CPR * 16);
        typedef short short8_t __attribute__((ext_vector_type(8)));
        short8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bfr[nt] = __builtin_bit_cast(bf16x8, v);
      }
#pragma unroll
      for (int mt = 0; mt < Cfg::MT; mt++)
#pragma unroll
        for (int nt = 0; nt < Cfg::NT; nt++)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[nt], af[mt], acc[mt][nt], 0, 0, 0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }

  // ---- epilogue: accumulator register e of lane l holds C[row = l%32][col = (e/4)*8 + (l/32)*4 + e%4]
  const int c_row = wm * Cfg::WTM + (lane & 31);
  const int c_col = wn * Cfg::WTN + (lane >> 5) * 4;
#pragma unroll
  for (int mt = 0; mt < Cfg::MT; mt++) {
    int row = c_row + mt * 32;
    if (row < rows) {
      bf16_t* crow = c + (long)row * ldc;
#pragma unroll
      for (int nt = 0; nt < Cfg::NT; nt++) {
#pragma unroll
        for (int g = 0; g < 4; g++) {
          int col = c_col + nt * 32 + g * 8;
          if (col < cols) {  // cols % 8 == 0 and col % 4 == 0: a 4-wide group is all in or all out
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; e++) o[e] = (bf16_t)acc[mt][nt][g * 4 + e];
            *(bf16x4*)(crow + col) = o;
          }
        }
      }
    }
  }
}

}  // namespace tl
