// Prefill compaction as a matrix-core GEMM (paper Sec. 3.1: Kbar = K D_k^T for given D_k).
//
//   C[b, row0 + t, j] = sum_c X[b, t, c] * Bm[b][j, c]         X [n, HD], Bm [r, HD], C [T_cap, r]
//
// The kernel is a general "NT" product C[m, j] = sum_k A[m, k] B[j, k] of two 16-bit matrices
// that are contiguous along the contraction axis (leading dimensions and batch strides of their
// own, fp32 accumulation, output in the storage type, as int8 codes + scales, or in fp32); the
// compression step's randomized SVD (bases.hip) uses it for its large products as well.
//
// Both operands are contiguous along the contraction axis, so tiles go HBM -> LDS with
// direct-to-LDS 16-byte loads and come back out as MFMA operands with one ds_read_b128 each.
// A workgroup (8 waves, 4 x 2) owns a 256-token x 128-column tile and walks the hidden axis
// in blocks of 64 through a three-stage LDS ring (two stages in flight while one is multiplied,
// one barrier per block); each wave holds a 64 x 64 accumulator as 2 x 2 MFMA 32x32x16 tiles.
// The LDS image of a tile is [row][8 chunks of 16 B] with the chunk index XOR-ed by (row/2 & 7): the loads pick their global source accordingly, and eight
// consecutive rows of one chunk column then sit in eight different bank groups.
// The MFMA computes the transposed tile (basis rows as the A operand), so a lane ends up with
// four consecutive output columns of one token; the tile is rounded to the storage type,
// staged in LDS and leaves in 16-byte row segments (or, for int8 output, as per-token
// per-64-column codes and fp16 scales).
// Workgroups are numbered so that the eight XCDs (round-robin over consecutive workgroup
// ids) each work through their own run of (sequence, token tile) pairs with the column
// tiles innermost: a token tile is fetched from HBM once and a sequence's basis stays in
// that XCD's L2.
#include "ap_common.hpp"

namespace ap {
namespace {

constexpr int kBM = 256;   // tokens per tile
constexpr int kBN = 128;   // output columns (basis rows) per tile
constexpr int kBK = 64;    // hidden elements per stage
constexpr int kStageBytes = (kBM + kBN) * kBK * 2;   // 48 KiB
constexpr int kStages = 3;
constexpr int kThreads = 512;
constexpr int kEpiPitch = kBN + 8;                   // 16-bit elements per staged output row

template <class Tag> struct Mfma32;
template <> struct Mfma32<F16Tag> {
  static __device__ __forceinline__ f32x16_t run(u32x4_t a, u32x4_t b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a),
                                                  __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
  }
};
template <> struct Mfma32<BF16Tag> {
  static __device__ __forceinline__ f32x16_t run(u32x4_t a, u32x4_t b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
};

__device__ __forceinline__ void dma16(const void* gsrc, void* lds_uniform) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gsrc,
                                   (__attribute__((address_space(3))) void*)lds_uniform, 16, 0, 0);
}

struct GemmParams {
  const uint16_t* X;        // A [n][lda] per batch item (x_bstride elements apart)
  const uint16_t* Bm;       // B [r][ldb] per batch item (bstride elements apart, 0 = shared)
  int64_t bstride, x_bstride, c_bstride, s_bstride;
  void* C;                  // [n][ldc] per batch item, already offset to its first row
  uint16_t* scale;          // int8 output: [n][r / 64] per batch item, already offset
  int n, HD, r, out_kind;   // rows of A, contraction length, rows of B; 0 = 16-bit, 1 = int8, 2 = fp32
  int lda, ldb, ldc;
  int MT, NT, G;            // token tiles, column tiles, workgroups in all
  // a second projection of the same shape in the same launch (keys and values of one prefill):
  // tiles G1 .. G-1 belong to it.  One launch of twice the tiles loses half as much to the last,
  // partly filled round of workgroups as two launches do.
  const uint16_t* X2;
  const uint16_t* Bm2;
  void* C2;
  uint16_t* scale2;
  int G1;
};

template <class Tag>
__global__ void __launch_bounds__(kThreads) compact_gemm(const GemmParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  // XCD-aware numbering: consecutive workgroup ids go to different XCDs
  const int per_xcd = (p.G + 7) >> 3;
  int logical = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (logical >= p.G) return;
  const bool second = logical >= p.G1;
  if (second) logical -= p.G1;
  const int nt = logical % p.NT;
  const int mt = (logical / p.NT) % p.MT;
  const int b = logical / (p.NT * p.MT);
  const int m0 = mt * kBM, n0 = nt * kBN;
  const char* Xb = (const char*)((second ? p.X2 : p.X) + (size_t)b * p.x_bstride);
  const char* Bb = (const char*)((second ? p.Bm2 : p.Bm) + (size_t)b * p.bstride);
  char* const Cout = (char*)(second ? p.C2 : p.C) +
                     (size_t)b * p.c_bstride * (p.out_kind == 0 ? 2 : (p.out_kind == 1 ? 1 : 4));
  uint16_t* const Sout = (second ? p.scale2 : p.scale) + (size_t)b * p.s_bstride;

  // ---- direct-to-LDS loads: per stage 32 KiB of X rows then 16 KiB of basis rows; wave w
  //      issues 1-KiB blocks 4w .. 4w+3 of the former and 2w, 2w+1 of the latter.  Block j,
  //      lane i -> LDS chunk P = 64 j + i, holding (row P>>3, hidden chunk (P&7) ^ (row/2 & 7)).
  uint32_t srcA[4], srcB[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int P = (4 * w + i) * 64 + lane;
    const int row = P >> 3, kc = (P & 7) ^ ((row >> 1) & 7);
    int ra = m0 + row;  ra = ra < p.n ? ra : p.n - 1;        // rows past the end: finite duplicates
    srcA[i] = ((uint32_t)ra * (uint32_t)p.lda + (uint32_t)kc * 8u) * 2u;
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int P = (2 * w + i) * 64 + lane;
    const int row = P >> 3, kc = (P & 7) ^ ((row >> 1) & 7);
    int rb = n0 + row;  rb = rb < p.r ? rb : p.r - 1;
    srcB[i] = ((uint32_t)rb * (uint32_t)p.ldb + (uint32_t)kc * 8u) * 2u;
  }
  auto issue = [&](int stage, int kb) {
    char* sA = smem + stage * kStageBytes + (4 * w) * 1024;
    char* sB = smem + stage * kStageBytes + kBM * kBK * 2 + (2 * w) * 1024;
    const uint32_t koff = (uint32_t)kb * (kBK * 2);
#pragma unroll
    for (int i = 0; i < 4; ++i) dma16(Xb + (srcA[i] + koff), sA + i * 1024);
#pragma unroll
    for (int i = 0; i < 2; ++i) dma16(Bb + (srcB[i] + koff), sB + i * 1024);
  };

  // ---- MFMA operands: wave (wn, wm) owns columns 64 wn .. and tokens 64 wm ..; operand row
  //      = lane & 31, hidden chunk of k-step ks = 2 ks + (lane >> 5)
  const int wn = w & 1, wm = w >> 1;                       // wm = 0 .. 3
  const int orow = lane & 31, ohalf = lane >> 5;
  uint32_t offN[2], offM[2], kx[4];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    offN[i] = (uint32_t)(kBM * kBK * 2 + (wn * 64 + i * 32 + orow) * 128);
    offM[i] = (uint32_t)((wm * 64 + i * 32 + orow) * 128);
  }
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) kx[ks] = (uint32_t)(((2 * ks + ohalf) ^ ((orow >> 1) & 7)) * 16);

  f32x16_t acc[2][2];      // [column tile][token tile]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // Software pipeline over the hidden axis, per 64-element block kb (stage kb % 3):
  //   wait:    this wave's loads of block kb+1 have landed, its operands of block kb are in
  //            registers
  //   barrier: the same holds for every wave, so block kb+1 may be read and the stage of
  //            block kb (fully consumed into registers) may be refilled with block kb+3
  //   then:    request block kb+3, read the operands of block kb+1 into the other register
  //            set, and multiply block kb -- the LDS reads and the loads run under the MFMAs.
  const int nk = p.HD / kBK;
  auto read_ops = [&](int stage, u32x4_t (&fa)[4][2], u32x4_t (&fb)[4][2]) {
    const char* st = smem + stage * kStageBytes;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[ks][i] = *(const u32x4_t*)(st + offN[i] + kx[ks]);
        fb[ks][i] = *(const u32x4_t*)(st + offM[i] + kx[ks]);
      }
  };
  auto multiply = [&](const u32x4_t (&fa)[4][2], const u32x4_t (&fb)[4][2]) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = Mfma32<Tag>::run(fa[ks][i], fb[ks][j], acc[i][j]);
  };
  // Wait for this wave's LDS reads and tell the compiler that the operand registers are
  // settled (it cannot see through the hand-placed wait and would otherwise add its own,
  // after the NEXT block's reads have been issued, which would serialise them with the MFMAs).
  auto settle = [&](u32x4_t (&fa)[4][2], u32x4_t (&fb)[4][2]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(fa[0][0]), "+v"(fa[0][1]), "+v"(fa[1][0]), "+v"(fa[1][1]), "+v"(fa[2][0]),
                   "+v"(fa[2][1]), "+v"(fa[3][0]), "+v"(fa[3][1]), "+v"(fb[0][0]), "+v"(fb[0][1]),
                   "+v"(fb[1][0]), "+v"(fb[1][1]), "+v"(fb[2][0]), "+v"(fb[2][1]), "+v"(fb[3][0]),
                   "+v"(fb[3][1])
                 :
                 : "memory");
  };
  u32x4_t fa0[4][2], fb0[4][2], fa1[4][2], fb1[4][2];
  issue(0, 0);
  if (nk > 1) issue(1, 1);
  if (nk > 2) issue(2, 2);
  // block 0: six loads per block and wave; later blocks may stay in flight
  if (nk > 2) asm volatile("s_waitcnt vmcnt(12)" ::: "memory");
  else if (nk > 1) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  read_ops(0, fa0, fb0);
  auto step = [&](int kb, u32x4_t (&fa_cur)[4][2], u32x4_t (&fb_cur)[4][2],
                  u32x4_t (&fa_nxt)[4][2], u32x4_t (&fb_nxt)[4][2]) {
    // outstanding loads of this wave at this point: blocks kb+1 and kb+2 (where they exist)
    if (kb + 2 < nk) asm volatile("s_waitcnt vmcnt(6)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    settle(fa_cur, fb_cur);
    asm volatile("s_barrier" ::: "memory");
    if (kb + 3 < nk) issue(kb % kStages, kb + 3);
    if (kb + 1 < nk) read_ops((kb + 1) % kStages, fa_nxt, fb_nxt);
    __builtin_amdgcn_sched_barrier(0);     // keep the requests ahead of the products
    multiply(fa_cur, fb_cur);
  };
  for (int kb = 0; kb < nk; kb += 2) {
    step(kb, fa0, fb0, fa1, fb1);
    if (kb + 1 < nk) step(kb + 1, fa1, fb1, fa0, fb0);
  }
  __syncthreads();                                         // the ring becomes the output staging area

  if (p.out_kind == 2) {
    // ---- fp32 output: stage [token][column] as floats, leave in 16-byte row segments
    constexpr int kPitch32 = kBN + 4;
    float* epf = (float*)smem;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
          const int col = wn * 64 + i * 32 + 8 * blk + 4 * ohalf;
          const int tok = wm * 64 + j * 32 + orow;
          const f32x4_t v = {acc[i][j][4 * blk + 0], acc[i][j][4 * blk + 1], acc[i][j][4 * blk + 2],
                             acc[i][j][4 * blk + 3]};
          *(f32x4_t*)(epf + tok * kPitch32 + col) = v;
        }
    __syncthreads();
    const int c4 = tid & 31, colf = n0 + c4 * 4;
#pragma unroll 1
    for (int pass = 0; pass < kBM / 16; ++pass) {
      const int tok = pass * 16 + (tid >> 5);
      const int t = m0 + tok;
      if (t < p.n && colf < p.r)      // r is a multiple of 8 on this path: whole 16-byte pieces
        *(f32x4_t*)((float*)Cout + (size_t)t * p.ldc + colf) = *(const f32x4_t*)(epf + tok * kPitch32 + c4 * 4);
    }
    return;
  }
  // ---- epilogue: round to the storage type, stage [token][column] in LDS
  uint16_t* epi = (uint16_t*)smem;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        const int col = wn * 64 + i * 32 + 8 * blk + 4 * ohalf;
        const int tok = wm * 64 + j * 32 + orow;
        u32x2_t v;
        v[0] = pack2(acc[i][j][4 * blk + 0], acc[i][j][4 * blk + 1], Tag{});
        v[1] = pack2(acc[i][j][4 * blk + 2], acc[i][j][4 * blk + 3], Tag{});
        *(u32x2_t*)(epi + tok * kEpiPitch + col) = v;
      }
  __syncthreads();
  const int c8 = tid & 15;
  const int col = n0 + c8 * 8;
#pragma unroll 1
  for (int pass = 0; pass < kBM / 32; ++pass) {
    const int tok = pass * 32 + (tid >> 4);
    const int t = m0 + tok;
    const u32x4_t v = *(const u32x4_t*)(epi + tok * kEpiPitch + c8 * 8);
    const bool live = t < p.n && col < p.r;
    const size_t row = (size_t)t;
    if (p.out_kind == 0) {
      if (live) *(u32x4_t*)((uint16_t*)Cout + row * p.ldc + col) = v;
    } else {
      // int8 format: amax over the 64-column block (8 lanes x 8 values), fp16 scale, codes
      float x[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) { x[2 * e] = lo_to_f32(v[e], F16Tag{}); x[2 * e + 1] = hi_to_f32(v[e], F16Tag{}); }
      float amax = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(x[e]));
#pragma unroll
      for (int o = 1; o < 8; o <<= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
      const _Float16 sh = (_Float16)(amax / 127.0f);       // IEEE divide, RNE to fp16
      const float s = (float)sh;
      uint32_t lo = 0, hi = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float q = 0.f;
        if (s != 0.f) q = fminf(fmaxf(rintf(x[e] / s), -127.f), 127.f);
        const uint32_t byte = (uint32_t)(int)q & 0xffu;
        if (e < 4) lo |= byte << (8 * e); else hi |= byte << (8 * (e - 4));
      }
      if (live) {
        u32x2_t cw = {lo, hi};
        *(u32x2_t*)((int8_t*)Cout + row * p.ldc + col) = cw;
        if ((c8 & 7) == 0) Sout[row * (p.r / AP_QBLOCK) + (col >> 6)] = __builtin_bit_cast(uint16_t, sh);
      }
    }
  }
}

template <class Tag>
ap_status run_gemm(const NtGemmArgs& a, const NtGemmArgs* a2) {
  GemmParams p{};
  p.X = (const uint16_t*)a.A;
  p.Bm = (const uint16_t*)a.Bm;
  p.bstride = a.b_bstride; p.x_bstride = a.a_bstride; p.c_bstride = a.c_bstride; p.s_bstride = a.s_bstride;
  p.C = a.C;
  p.scale = (uint16_t*)a.scale;
  p.n = a.M; p.HD = a.K; p.r = a.N;
  p.lda = a.lda; p.ldb = a.ldb; p.ldc = a.ldc;
  p.out_kind = a.out_kind;
  p.MT = (a.M + kBM - 1) / kBM;
  p.NT = (a.N + kBN - 1) / kBN;
  const int64_t G1 = (int64_t)a.batch * p.MT * p.NT;
  const int64_t G = a2 ? 2 * G1 : G1;
  AP_REQUIRE(G <= (1 << 28), AP_ERR_UNSUPPORTED, "matrix product: too many tiles");
  p.G = (int)G;
  p.G1 = (int)G1;
  if (a2) {
    p.X2 = (const uint16_t*)a2->A;
    p.Bm2 = (const uint16_t*)a2->Bm;
    p.C2 = a2->C;
    p.scale2 = (uint16_t*)a2->scale;
  }
  const int grid = ((p.G + 7) / 8) * 8;
  auto kern = compact_gemm<Tag>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kStages * kStageBytes);
    if (e != hipSuccess) {
      set_error("hipFuncSetAttribute: %s", hipGetErrorString(e));
      return AP_ERR_HIP;
    }
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), kStages * kStageBytes, a.stream, p);
  return check_launch("matrix product");
}

NtGemmArgs nt_args_of(const CompactArgs& a) {
  NtGemmArgs g{};
  g.A = a.X; g.a_bstride = (int64_t)a.n * a.HD; g.lda = a.HD;
  g.Bm = a.Bm; g.b_bstride = a.basis_batch_stride; g.ldb = a.HD;
  const size_t esz = a.dt_out == AP_I8 ? 1 : 2;
  g.C = (char*)a.C + (size_t)a.row0 * a.r * esz; g.c_bstride = (int64_t)a.T_cap * a.r; g.ldc = a.r;
  g.scale = a.scale ? (uint16_t*)a.scale + (size_t)a.row0 * (a.r / AP_QBLOCK) : nullptr;
  g.s_bstride = (int64_t)a.T_cap * (a.r / AP_QBLOCK);
  g.batch = a.B; g.M = a.n; g.N = a.r; g.K = a.HD;
  g.dt = a.dt_in; g.out_kind = a.dt_out == AP_I8 ? 1 : 0; g.stream = a.stream;
  return g;
}

}  // namespace

// The matrix-core path takes 16-bit inputs whose hidden axis is a multiple of 64 and whose
// per-sequence byte offsets fit 32 bits; anything else stays on the row kernel.
bool compact_gemm_applies(const CompactArgs& a) {
  if (a.dt_in != AP_F16 && a.dt_in != AP_BF16) return false;
  if (a.n < 32 || a.HD % kBK != 0 || a.r % 8 != 0) return false;
  if ((int64_t)a.n * a.HD * 2 >= (1ll << 32) || (int64_t)a.r * a.HD * 2 >= (1ll << 32)) return false;
  return true;
}

ap_status launch_compact_gemm(const CompactArgs& a, const CompactArgs* second) {
  const NtGemmArgs g = nt_args_of(a);
  if (!second) return launch_gemm_nt(g, nullptr);
  const NtGemmArgs g2 = nt_args_of(*second);
  return launch_gemm_nt(g, &g2);
}

// C[b][m, j] = sum_k A[b][m, k] B[b][j, k]: K a multiple of 64, N a multiple of 8, 16-byte aligned
// rows, per-item byte offsets below 4 GiB.  `second`: another product of the same shape in the
// same launch (only its A, Bm, C, scale are read).
ap_status launch_gemm_nt(const NtGemmArgs& a, const NtGemmArgs* second) {
  AP_REQUIRE(a.K % kBK == 0 && a.N % 8 == 0 && a.lda % 8 == 0 && a.ldb % 8 == 0 && a.M > 0 && a.N > 0,
             AP_ERR_UNSUPPORTED, "matrix product: K %% 64, N %% 8 and 16-byte aligned rows are required");
  AP_REQUIRE((int64_t)a.M * a.lda * 2 < (1ll << 32) && (int64_t)a.N * a.ldb * 2 < (1ll << 32), AP_ERR_UNSUPPORTED,
             "matrix product: one operand must stay below 4 GiB");
  return a.dt == AP_F16 ? run_gemm<F16Tag>(a, second) : run_gemm<BF16Tag>(a, second);
}

}  // namespace ap
