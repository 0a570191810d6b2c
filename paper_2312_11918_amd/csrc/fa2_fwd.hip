// FlashAttention-2 forward pass for gfx950 (MI355X, CDNA4): kernel and C ABI of libfa2.
//
// Follows Algorithm 2 of arXiv 2312.11918 (tile of query rows per workgroup, loop over K/V tiles,
// GEMM-I, online softmax, GEMM-II, final division by the row sum) with a data flow designed for
// 64-lane wavefronts and MFMA instead of the paper's Hopper TMA/WGMMA pipeline:
//
//  * Both products are computed TRANSPOSED, S^T = K Q^T and O^T = V^T P^T, with
//    v_mfma_f32_32x32x16.  In the 32x32 accumulator layout a lane owns one column, so with the
//    transposed products every lane owns ONE QUERY: the row maximum and row sum of Algorithm 2 are
//    in-lane reductions plus a single exchange between lane l and lane l+32, the rescale factor
//    exp(m_old - m_new) is a per-lane scalar, and the S^T accumulator registers, rounded to 16 bit,
//    already have the register layout of the B operand of the second product (Section 4.2 of the
//    paper solves the same accumulator-to-operand problem for WGMMA by re-indexing the fragment).
//    The only price is that the key index inside a 16-key MFMA step is permuted; a contraction
//    does not care about the order of its terms, and V is read from LDS with the same permutation.
//  * V is the operand whose contraction index (the key) is not contiguous in memory (Section 4.1
//    of the paper takes a transposed shared-memory view).  Here V stays row-major in LDS and is
//    read with ds_read_b64_tr_b16, the LDS transpose load of gfx950.
//  * K/V tiles are double-buffered in LDS and the next tile's global loads are issued before the
//    current tile's MFMAs (the copy/GEMM overlap of Section 6, without TMA or mbarriers).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fa2.h"

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;            // wavefronts per workgroup
constexpr int kThreads = kWaves * 64;
constexpr int kBr = 32 * kWaves;     // query rows per workgroup (32 per wavefront)
constexpr int kBc = 64;              // keys per K/V tile
constexpr int kXcds = 8;             // accelerator complex dies; workgroup i is dispatched to XCD i % 8

// Element-type specifics: the MFMA flavour and the fp32 -> 16-bit pack (round to nearest even).
template <int DT> struct Elem;
template <> struct Elem<FA2_FP16> {
  static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f16x2 r = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, r);
  }
};
template <> struct Elem<FA2_BF16> {
  static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    bf16x2 r = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, r);
  }
};

// Value held by the partner lane (l ^ 32): v_permlane32_swap exchanges the upper half of one
// register with the lower half of another, which leaves each half's value broadcast in one result.
__device__ __forceinline__ float max_with_partner_half(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}
__device__ __forceinline__ float sum_with_partner_half(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}

// LDS transpose load: within each group of 16 lanes the 16 x 4 block of 16-bit elements addressed
// by the lanes (lane p supplies 4 consecutive elements) is transposed, so that lane i receives
// element (i % 4) of lanes i/4, 4 + i/4, 8 + i/4 and 12 + i/4.
__device__ __forceinline__ u32x2 lds_read_tr16(const uint16_t* p) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
  return __builtin_bit_cast(u32x2, v);
}

// Row strides of the LDS tiles in 16-bit elements.  K is read with 16-byte loads, lane = key row:
// a stride of (row bytes + 16) spreads 16 consecutive rows over all banks.  V is read with the
// transpose load, 8 key rows x 64 bytes per instruction: a stride of 64 bytes modulo 256 puts
// four consecutive rows side by side across the 64 banks.
template <int D> struct Lds {
  static constexpr int kKStride = D + 8;
  static constexpr int kVStride = D + 32;
  static constexpr int kKTile = kBc * kKStride;
  static constexpr int kVTile = kBc * kVStride;
};

template <int DT, int D>
__global__ __launch_bounds__(kThreads, 2) void fa2_fwd_kernel(const uint16_t* __restrict__ Q,
                                                              const uint16_t* __restrict__ K,
                                                              const uint16_t* __restrict__ V,
                                                              uint16_t* __restrict__ O, float* __restrict__ LSE,
                                                              int H, int N, float scale_log2e, int n_qtiles,
                                                              int total_tiles) {
  using E = Elem<DT>;
  using L = Lds<D>;
  constexpr int kKSteps = D / 16;   // MFMA steps along d for S^T = K Q^T
  constexpr int kDBlocks = D / 32;  // 32-row blocks of O^T
  constexpr int kChunksPerRow = D / 8;                        // 16-byte chunks per K/V row
  constexpr int kChunksPerThread = kBc * kChunksPerRow / kThreads;

  __shared__ __attribute__((aligned(16))) uint16_t k_lds[2][L::kKTile];
  __shared__ __attribute__((aligned(16))) uint16_t v_lds[2][L::kVTile];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r = lane & 31;   // column of the 32x32 MFMA tile owned by this lane = query within the wave
  const int hh = lane >> 5;  // which half of the wavefront

  // Q-tile scheduling (Algorithm 2's outer loop, parallel over workgroups).  Workgroups are dealt
  // round-robin to the 8 XCDs, each with its own L2: give every XCD a contiguous range of tiles so
  // that the Q tiles of one head, which all stream the same K and V, share one L2.
  int tile;
  {
    const int wg = blockIdx.x;
    const int per = total_tiles / kXcds, rem = total_tiles % kXcds;
    const int xcd = wg % kXcds, idx = wg / kXcds;
    tile = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  const int bh = tile / n_qtiles;
  const int qt = tile - bh * n_qtiles;
  const int b = bh / H;
  const int h = bh - b * H;

  const size_t row_stride = (size_t)H * D;                          // elements between consecutive tokens
  const size_t head_base = ((size_t)b * N * H + (size_t)h) * D;     // element (b, 0, h, 0)
  const int q_row = qt * kBr + wave * 32 + r;

  // Q_i fragment, held in registers for the whole loop: B operand of S^T = K Q^T.
  u32x4 qf[kKSteps];
  {
    const uint16_t* qp = Q + head_base + (size_t)q_row * row_stride + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks) qf[ks] = *reinterpret_cast<const u32x4*>(qp + 16 * ks);
  }

  // Staging of one K/V tile: thread t moves 16-byte chunks t, t+256, ... of the tile.
  u32x4 kreg[kChunksPerThread], vreg[kChunksPerThread];
  auto load_tile = [&](int j) {
    const size_t tile_base = head_base + (size_t)j * kBc * row_stride;
#pragma unroll
    for (int i = 0; i < kChunksPerThread; ++i) {
      const int c = tid + i * kThreads;
      const int row = c / kChunksPerRow, col = c % kChunksPerRow;
      const size_t off = tile_base + (size_t)row * row_stride + col * 8;
      kreg[i] = *reinterpret_cast<const u32x4*>(K + off);
      vreg[i] = *reinterpret_cast<const u32x4*>(V + off);
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < kChunksPerThread; ++i) {
      const int c = tid + i * kThreads;
      const int row = c / kChunksPerRow, col = c % kChunksPerRow;
      *reinterpret_cast<u32x4*>(&k_lds[buf][row * L::kKStride + col * 8]) = kreg[i];
      *reinterpret_cast<u32x4*>(&v_lds[buf][row * L::kVStride + col * 8]) = vreg[i];
    }
  };

  // Accumulators of Algorithm 2: O^T (fp32), running rowmax (kept unscaled, and scaled by
  // scale*log2(e) as the reference point of the exponentials) and running rowsum.  Each half of the
  // wavefront keeps the partial rowsum of its own keys; the two are added in the epilogue.
  f32x16 ot[kDBlocks];
#pragma unroll
  for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) ot[db][v] = 0.f;
  float m_run = -INFINITY;   // running rowmax of the unscaled logits q.k
  float mc_run = -INFINITY;  // the same times scale*log2(e)
  float l_run = 0.f;

  const int n_tiles = N / kBc;
  load_tile(0);
  store_tile(0);
  __syncthreads();

  // Per-lane LDS element offsets of the operand reads.
  const int k_off = r * L::kKStride + 8 * hh;
  const int v_off = (4 * hh + ((lane & 15) >> 2)) * L::kVStride + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

  for (int j = 0; j < n_tiles; ++j) {
    const int buf = j & 1;
    if (j + 1 < n_tiles) load_tile(j + 1);  // in flight during this tile's MFMAs

    // GEMM-I (transposed): S^T[key][query] for 2 blocks of 32 keys.
    f32x16 st[kBc / 32];
#pragma unroll
    for (int kb = 0; kb < kBc / 32; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) st[kb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < kKSteps; ++ks) {
        const u32x4 kf = *reinterpret_cast<const u32x4*>(&k_lds[buf][k_off + kb * 32 * L::kKStride + ks * 16]);
        st[kb] = E::mfma(kf, qf[ks], st[kb]);
      }
    }

    // Online softmax for this lane's query.  The maximum is taken on the unscaled logits (valid for
    // scale > 0) and the scale is folded into the exponent: exp(scale*(s-m)) = exp2(s*c - m*c).
    float mx = st[0][0];
#pragma unroll
    for (int kb = 0; kb < kBc / 32; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, st[kb][v]);
    mx = max_with_partner_half(mx);
    const float m_new = fmaxf(m_run, mx);
    const float mc_new = m_new * scale_log2e;
    const float alpha = __builtin_amdgcn_exp2f(mc_run - mc_new);  // exp(m_old - m_new); 0 on the first tile
    m_run = m_new;
    mc_run = mc_new;

    float rowsum = 0.f;
    u32x4 pf[kBc / 16];
#pragma unroll
    for (int kb = 0; kb < kBc / 32; ++kb) {
      float p[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        p[v] = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kb][v], scale_log2e, -mc_new));
        rowsum += p[v];
      }
      // P~ rounded to 16 bit: registers 8t..8t+7 of a 32-key block are the 8 B-operand slots of MFMA step t.
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        pf[kb * 2 + t] = u32x4{E::pack2(p[8 * t + 0], p[8 * t + 1]), E::pack2(p[8 * t + 2], p[8 * t + 3]),
                               E::pack2(p[8 * t + 4], p[8 * t + 5]), E::pack2(p[8 * t + 6], p[8 * t + 7])};
      }
    }
    l_run = alpha * l_run + rowsum;
#pragma unroll
    for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) ot[db][v] *= alpha;

    // GEMM-II (transposed): O^T[d][query] += V^T P^T.  Slot i of lane-half hh in step t is key
    // 16t + 8(i/4) + 4hh + i%4, the key of accumulator register 8t+i of GEMM-I.
#pragma unroll
    for (int t = 0; t < kBc / 16; ++t) {
#pragma unroll
      for (int db = 0; db < kDBlocks; ++db) {
        const uint16_t* vp = &v_lds[buf][v_off + t * 16 * L::kVStride + db * 32];
        const u32x2 lo = lds_read_tr16(vp);
        const u32x2 hi = lds_read_tr16(vp + 8 * L::kVStride);
        ot[db] = E::mfma(u32x4{lo[0], lo[1], hi[0], hi[1]}, pf[t], ot[db]);
      }
    }

    // The other buffer was last read during tile j-1; every wavefront has passed the barrier that
    // ended that iteration, so it can be overwritten now.
    if (j + 1 < n_tiles) store_tile(buf ^ 1);
    __syncthreads();
  }

  // Epilogue: O_i = O_i / rowsum, LSE_i = m_i + ln(rowsum) (natural log, scaled logits).
  const float l_tot = sum_with_partner_half(l_run);
  const float inv_l = 1.0f / l_tot;
  uint16_t* op = O + head_base + (size_t)q_row * row_stride + 4 * hh;
#pragma unroll
  for (int db = 0; db < kDBlocks; ++db) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      // accumulator registers 4g..4g+3 hold d = 32 db + 8 g + 4 hh + (0..3) of this lane's query
      u32x2 w = {E::pack2(ot[db][4 * g + 0] * inv_l, ot[db][4 * g + 1] * inv_l),
                 E::pack2(ot[db][4 * g + 2] * inv_l, ot[db][4 * g + 3] * inv_l)};
      *reinterpret_cast<u32x2*>(op + db * 32 + g * 8) = w;
    }
  }
  if (LSE != nullptr && hh == 0) {
    LSE[((size_t)b * H + h) * N + q_row] = mc_run * 0.69314718055994530942f + __builtin_logf(l_tot);
  }
}

template <int DT, int D>
int launch(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int N, float scale,
           hipStream_t stream) {
  const int n_qtiles = N / kBr;
  const long long total = (long long)B * H * n_qtiles;
  if (total > 0x7fffffffLL) return FA2_ERR_UNSUPPORTED;
  const float scale_log2e = scale * 1.44269504088896340736f;
  hipLaunchKernelGGL((fa2_fwd_kernel<DT, D>), dim3((unsigned)total), dim3(kThreads), 0, stream,
                     static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
                     static_cast<const uint16_t*>(V), static_cast<uint16_t*>(O), LSE, H, N, scale_log2e, n_qtiles,
                     (int)total);
  return hipGetLastError() == hipSuccess ? FA2_OK : FA2_ERR_LAUNCH;
}

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

extern "C" int fa2_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int N, int d,
                       float scale, int dtype, void* stream) {
  // All validation happens before the first HIP call: an error launches nothing.
  if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr) return FA2_ERR_INVALID_ARG;
  if (B <= 0 || H <= 0 || N <= 0 || d <= 0) return FA2_ERR_INVALID_ARG;
  if (!(scale > 0.0f) || !(scale <= 3.0e38f)) return FA2_ERR_INVALID_ARG;  // rejects NaN, inf, <= 0
  if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) || !aligned(LSE, 4))
    return FA2_ERR_INVALID_ARG;
  if (dtype != FA2_FP16 && dtype != FA2_BF16) return FA2_ERR_UNSUPPORTED;
  if (d != 64 && d != 128) return FA2_ERR_UNSUPPORTED;
  if (N % kBr != 0) return FA2_ERR_UNSUPPORTED;
  // element offsets are computed in 64 bits; the row index b*N+n must still fit the tile arithmetic
  if ((long long)B * N > 0x7fffffffLL) return FA2_ERR_UNSUPPORTED;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == FA2_FP16) {
    return d == 64 ? launch<FA2_FP16, 64>(Q, K, V, O, LSE, B, H, N, scale, s)
                   : launch<FA2_FP16, 128>(Q, K, V, O, LSE, B, H, N, scale, s);
  }
  return d == 64 ? launch<FA2_BF16, 64>(Q, K, V, O, LSE, B, H, N, scale, s)
                 : launch<FA2_BF16, 128>(Q, K, V, O, LSE, B, H, N, scale, s);
}

extern "C" const char* fa2_strerror(int code) {
  switch (code) {
    case FA2_OK: return "success";
    case FA2_ERR_INVALID_ARG: return "invalid argument (NULL or misaligned pointer, non-positive size, or scale not finite and > 0)";
    case FA2_ERR_UNSUPPORTED: return "unsupported problem (d must be 64 or 128, N a multiple of 128, dtype fp16 or bf16)";
    case FA2_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    default: return "unknown fa2 error code";
  }
}

extern "C" int fa2_version(void) { return 100; /* 0.1.0 */ }
