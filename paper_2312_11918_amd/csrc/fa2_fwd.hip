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
//  * K/V tiles are double-buffered (or held in a ring of four) in LDS and the next tiles' global loads are
//    issued before the current tile's MFMAs (the copy/GEMM overlap of Section 6, without TMA or mbarriers;
//    the producer/consumer hand-over is a barrier per tile in one tile shape and counters in LDS in the other).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <tuple>
#include <type_traits>
#include <utility>

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

constexpr int kWaves = 4;            // wavefronts per workgroup of the 128-row shape
constexpr int kBr = 32 * kWaves;     // query rows per workgroup (32 per wavefront)
constexpr int kBc = 64;              // keys per K/V tile
constexpr int kSpinLimit = 1 << 18;  // polls of the arrival count before a wavefront gives up (tens of milliseconds)
constexpr int kCUs = 256;            // compute units of the whole chip (tile-shape choice only)
constexpr int kXcds = 8;             // accelerator complex dies; workgroup i is dispatched to XCD i % 8
constexpr float kLazyLog2 = 8.0f;    // the rowmax reference moves only when exceeded by 2^8

// Element-type specifics: the MFMA flavour and the fp32 -> 16-bit pack (round to nearest even).
// Compile-time loop: calls f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N-1>{}).
template <int... I, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, static_cast<F&&>(f));
}

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
__device__ __forceinline__ float sum_with_partner_half(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}

// Maximum of two / three values as single instructions.  fmaxf() makes the compiler quiet possible
// signalling NaNs of every input first (one extra instruction each); inputs here are finite by contract.
__device__ __forceinline__ float max2_raw(float a, float b) {
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float max3_raw(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ __forceinline__ float max_with_partner_half_raw(float x) {
  uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return max2_raw(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}

// LDS transpose load: within each group of 16 lanes the 16 x 4 block of 16-bit elements addressed
// by the lanes (lane p supplies 4 consecutive elements) is transposed, so that lane i receives
// element (i % 4) of lanes i/4, 4 + i/4, 8 + i/4 and 12 + i/4.
__device__ __forceinline__ u32x2 lds_read_tr16(const uint16_t* p) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
  return __builtin_bit_cast(u32x2, v);
}

// LDS tile geometry.  A K or V tile is kBc rows of D 16-bit elements, stored row-major WITHOUT
// padding (the direct global->LDS loads write 1 KiB of consecutive LDS per wavefront instruction),
// with the 16-byte chunks of every row permuted by an XOR so that the operand reads are free of
// bank conflicts (the role of the paper's 128-byte shared-memory swizzle, Section 3.2):
//   K is read with 16-byte loads, lane = key row: 16 consecutive rows must land in 16 different
//     16-byte slots of the 256-byte bank period            -> chunk ^= f(row) over the whole period;
//   V is read with the transpose load, 4 key rows x 32 bytes per group of 16 lanes: the 4 rows must
//     land in different 64-byte quarters of the bank period -> chunk ^= g(row) << 2.
template <int D> struct Tile {
  static constexpr int kChunksPerRow = D / 8;                      // 16-byte chunks per row
  static constexpr int kElems = kBc * D;                           // elements per tile
  static constexpr int kLoadsPerWave = kElems * 2 / 1024 / kWaves; // 1 KiB wavefront loads per tile and wave
  static __device__ __forceinline__ int swz_k(int row) { return D >= 128 ? (row & 15) : ((row >> 1) & 7); }
  static __device__ __forceinline__ int swz_v(int row) { return (D >= 128 ? (row & 3) : ((row >> 1) & 1)) << 2; }
};

typedef __attribute__((address_space(3))) void* lds_void_ptr;
constexpr int kBufferFlags = 0x00020000;  // raw buffer descriptor word 3 for gfx9-family: 32-bit data format, no swizzle

// -------------------------------------------------------------------------------------------------
// Kernel with 32 query rows per wavefront.  kWv wavefronts form a workgroup (32*kWv rows); K and V tiles
// cycle through kNBuf LDS buffers each.  Two shapes are instantiated:
//   4 wavefronts, 2 buffers: 128 rows per workgroup, 2 workgroups per CU;
//   8 wavefronts, 4 buffers: 256 rows per workgroup, 1 workgroup per CU, global loads issued three
//                            tiles ahead and half the L2->LDS traffic per FLOP.  This shape has no barrier in
//                            its loop (arrival counters in LDS, see kFlagSync), takes `chain` Q tiles per
//                            workgroup over one running K/V stream (see kChain) and stores O as pieces of rows.
// Either way a SIMD runs two wavefronts, so one wavefront's softmax arithmetic overlaps the other's MFMAs.
// `total_tiles` is the number of workgroups; `chain` is 1 except for unmasked launches of the 8-wavefront shape.
//
// kCausal applies the optional mask of S (Section 2 of the paper: entries of S may be set to -inf before the
// softmax; here those with key index > query index).  A Q tile then stops at its diagonal: it visits
// (qt+1)*kNBuf K/V tiles instead of N/kBc, only the last kNBuf of them straddle the diagonal and need the
// element-wise mask, and a workgroup takes two Q tiles of one head, the p-th from the end and the p-th from the
// start, whose tile counts add up to the same number for every p.
//
// kRagged lifts the restriction to whole tiles: Nq query rows and Nk keys of any size >= 1.  Query rows past
// Nq-1 are computed from a copy of the last row and not stored; K/V rows past Nk-1 are staged as copies of
// the last row (finite data) and their columns of S are set to -inf in the last kNBuf tiles, the only ones
// that can hold them; the tile count is rounded up to a multiple of kNBuf (a padding tile is fully masked).
//
template <int DT, int D, int kWv, int kNBuf, bool kCausal, bool kRagged>
__global__ __launch_bounds__(kWv * 64, (kWv == 4 && D <= 128) ? 2 : 1) void fa2_fwd_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    uint16_t* __restrict__ O, float* __restrict__ LSE, int H, int Nq, int Nk, float scale_log2e, int n_qtiles,
    int total_tiles, int chain) {
  using E = Elem<DT>;
  using T = Tile<D>;
  using std::false_type;
  using std::true_type;
  static_assert(kNBuf == 2 || kNBuf == 4, "two or four LDS buffers per operand");
  constexpr int kRows = 32 * kWv;   // query rows per workgroup
  static_assert(kRows == kNBuf * kBc, "a Q tile spans exactly kNBuf K/V tiles (the causal tile count relies on it)");
  constexpr int kKSteps = D / 16;   // MFMA steps along d for S^T = K Q^T
  constexpr int kDBlocks = D / 32;  // 32-row blocks of O^T
  constexpr int kKBlocks = kBc / 32;  // 32-key blocks of S^T
  constexpr int kTSteps = kBc / 16;   // MFMA steps along the keys for O^T = V^T P^T
  constexpr int kSteps1 = kKBlocks * kKSteps;  // MFMAs of GEMM-I per tile
  constexpr int kSteps2 = kTSteps * kDBlocks;  // MFMAs of GEMM-II per tile
  constexpr int kRing = 4;                     // operand fragments in flight between LDS and the MFMAs
  constexpr int kLoadsPerWave = T::kElems * 2 / 1024 / kWv;  // 1 KiB wavefront loads per tile and wavefront
  constexpr bool kSplitRefill = kNBuf == 2 && D == 256;    // K and V refills issued as two separate bursts
  // The 8-wavefront shape has no barrier in its loop: its wavefronts count their arrivals at the end of every
  // iteration in LDS and go on as soon as all have finished the iteration BEFORE.  One barrier per tile would
  // start the two wavefronts of every SIMD in the same phase tile after tile, softmax against softmax and MFMAs
  // against MFMAs; with a tile of slack they drift apart and fill each other's gaps.
  constexpr bool kFlagSync = kWv == 8;
  // A workgroup of that shape takes `chain` Q tiles (under the causal mask: pairs of Q tiles, and the two of a
  // pair as well) one after the other, and the K/V stream runs on
  // from one to the next (after the last K/V tile of one comes the first of the next): only the first Q tile pays
  // for filling the ring, and with one workgroup per CU nothing else would cover that time.  The Q tiles of a
  // workgroup are spaced by the number of workgroups of its XCD, so that at any time the workgroups of an XCD
  // work on neighbouring Q tiles, a few heads whose K and V fit its L2, as they do without chaining.
  // The d = 256 kernel, also one workgroup per CU, chains in the same way when it runs on whole tiles.
  constexpr bool kChain = kFlagSync || (kWv == 4 && D == 256 && !kRagged);

  // The buffers are separate objects on purpose: the compiler then knows that a load in flight into one
  // buffer cannot alias the operand reads from another.  (With kNBuf == 2 the last two pairs are unused.)
  __shared__ __attribute__((aligned(1024))) uint16_t k_lds0[T::kElems];
  __shared__ __attribute__((aligned(1024))) uint16_t k_lds1[T::kElems];
  __shared__ __attribute__((aligned(1024))) uint16_t k_lds2[kNBuf == 4 ? T::kElems : 8];
  __shared__ __attribute__((aligned(1024))) uint16_t k_lds3[kNBuf == 4 ? T::kElems : 8];
  __shared__ __attribute__((aligned(1024))) uint16_t v_lds0[T::kElems];
  __shared__ __attribute__((aligned(1024))) uint16_t v_lds1[T::kElems];
  __shared__ __attribute__((aligned(1024))) uint16_t v_lds2[kNBuf == 4 ? T::kElems : 8];
  __shared__ __attribute__((aligned(1024))) uint16_t v_lds3[kNBuf == 4 ? T::kElems : 8];
  __shared__ uint32_t arrivals[4];  // kFlagSync: wavefronts that finished iteration j, counted in entry j % 4
  // kRowStores: 32 rows x 32 columns of O per wavefront, through which the result is turned from one query per
  // lane into whole 64-byte pieces of rows before it is stored: a lane-per-query store touches 64 rows per
  // instruction, and the epilogue of a Q tile then costs thousands of cycles that only partly hide behind the other
  // workgroups of the CU (measured: +2 % at N = 2048, +5...10 % at N <= 1024, more with one workgroup per CU)
  // (every kernel but one: the 128-row shape at d = 128 with both the causal mask and partial tiles has no
  // registers left for it)
  constexpr bool kRowStores = !(kWv == 4 && D == 128 && kCausal && kRagged);
  __shared__ __attribute__((aligned(16))) uint16_t o_slab[kRowStores ? kWv * 1024 : 8];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform, kept in a scalar register
  const int r = lane & 31;   // column of the 32x32 MFMA tile owned by this lane = query within the wave
  const int hh = lane >> 5;  // which half of the wavefront

  // Q-tile scheduling (Algorithm 2's outer loop, parallel over workgroups).  Workgroups are dealt
  // round-robin to the 8 XCDs, each with its own L2: give every XCD a contiguous range of tiles so
  // that the Q tiles of one head, which all stream the same K and V, share one L2.
  int tile, chain_stride = 0;  // kChain: the Q tile (pair) of chain step c is tile + c * chain_stride, over all heads
  {
    const int wg = blockIdx.x;
    const int per = total_tiles / kXcds, rem = total_tiles % kXcds;
    const int xcd = wg % kXcds, idx = wg / kXcds;
    const int first = xcd * per + (xcd < rem ? xcd : rem);  // first workgroup of this XCD's range
    if constexpr (kChain) {
      tile = first * chain + idx;
      chain_stride = per + (xcd < rem ? 1 : 0);
    } else {
      tile = first + idx;
    }
  }
  // Under the causal mask the work of Q tile qt grows like qt + 1, so a workgroup takes a PAIR of Q tiles of
  // one head, n_qtiles-1-p and then p, one after the other: every workgroup then does the same amount of
  // work (but for the unpaired middle tile when n_qtiles is odd).  total_tiles counts pairs in that case.
  const int n_items = kCausal ? (n_qtiles + 1) / 2 : n_qtiles;
  int bh = tile / n_items;                // batch entry * H + head (kChain: of the current pass)
  const int item = tile - bh * n_items;   // Q tile, or pair of Q tiles (kChain: first Q tile)
  // passes of this workgroup: Q tiles it works through.  A chain longer than 1 under the causal mask is only
  // launched when every pair is complete (n_qtiles even).
  const int n_pass = kCausal ? (chain > 1 ? 2 * chain : item != n_qtiles - 1 - item ? 2 : 1) : kChain ? chain : 1;
  int qt, q_row, n_tiles;  // set per pass

  const size_t row_stride = (size_t)H * D;                          // elements between consecutive tokens
  const size_t tile_stride = (size_t)kBc * row_stride;              // elements between consecutive K/V tiles
  // element (b, 0, h, 0) of Q and O / of K and V, for head index bh = b * H + h
  auto q_base_of = [&](int bh_) { return ((size_t)(bh_ / H) * Nq * H + (size_t)(bh_ % H)) * D; };
  auto kv_base_of = [&](int bh_) { return ((size_t)(bh_ / H) * Nk * H + (size_t)(bh_ % H)) * D; };
  size_t head_base = q_base_of(bh);

  // Q_i fragment, held in registers for the whole loop: B operand of S^T = K Q^T.
  u32x4 qf[kKSteps];

  // Direct global->LDS staging (buffer_load ... lds).  Wavefront w issues loads number w*kLoadsPerWave + i
  // of a tile; load n fills LDS bytes [1024 n, 1024 n + 1024) of the tile, lane l the 16-byte chunk
  // 64 n + l.  The chunk's row and (swizzled) position decide which global chunk the lane fetches.
  // Buffer descriptors (base, byte range) of this head's K and V rows: a raw buffer load takes a scalar
  // descriptor, a scalar tile offset and the 32-bit per-lane offset, and its range check turns any
  // offset past the last row into zeros instead of a fault.
  const uint32_t head_bytes = (uint32_t)(((size_t)(Nk - 1) * row_stride + D) * 2);
  auto rsrc_of = [&](const uint16_t* tensor, int bh_) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(tensor + kv_base_of(bh_)), 0, (int)head_bytes,
                                             kBufferFlags);
  };
  __amdgpu_buffer_rsrc_t k_rsrc = rsrc_of(K, bh), v_rsrc = rsrc_of(V, bh);
  // kChain: the head and Q tile of the next pass, whose first K/V tiles the last boundaries of this pass load
  // (their descriptors are made where they are used, not kept in scalar registers through the loop)
  int bh_next = 0, qt_next = 0;
  int stream_base = 0;  // kChain: K/V tiles streamed for the Q tiles this workgroup has finished
  bool more = false;    // kChain: another Q tile follows, so the stream goes on past tile n_tiles - 1
  const uint32_t tile_bytes = (uint32_t)(tile_stride * 2);
  const uint32_t row_bytes = (uint32_t)(row_stride * 2);
  // is_k is a compile-time tag: K and V tiles use different chunk swizzles.  The per-lane source offsets are
  // recomputed at every call (a few integer operations per tile) instead of being kept in registers.
  auto stage_in = [&](auto is_k, __amdgpu_buffer_rsrc_t rsrc, int j, uint16_t* lds_tile) __attribute__((always_inline)) {
    int lane = tid & 63;
    // d = 256 with partial tiles has no registers to spare for sixteen loop-invariant source offsets: keep them
    // from being hoisted out of the loop (they cost a few integer operations per load to recompute)
    if constexpr (D == 256 && kRagged) asm volatile("" : "+v"(lane));
    if (kRagged && (j + 1) * kBc > Nk) {
      // a tile with rows past the last key: those rows are filled with copies of the last key's row, so LDS
      // holds finite numbers everywhere (their columns of S are masked; 0 * finite = 0 in GEMM-II)
#pragma unroll
      for (int i = 0; i < kLoadsPerWave; ++i) {
        const int chunk = 64 * (wave * kLoadsPerWave + i) + lane;
        const int row = chunk / T::kChunksPerRow, pos = chunk % T::kChunksPerRow;
        const int swz = decltype(is_k)::value ? T::swz_k(row) : T::swz_v(row);
        const int row_g = min(j * kBc + row, Nk - 1);
        const uint32_t src = (uint32_t)row_g * row_bytes + 16u * (uint32_t)(pos ^ swz);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(lds_tile + 512 * (wave * kLoadsPerWave + i)), 16,
                                                 (int)src, 0, 0, 0);
      }
      return;
    }
#pragma unroll
    for (int i = 0; i < kLoadsPerWave; ++i) {
      const int chunk = 64 * (wave * kLoadsPerWave + i) + lane;
      const int row = chunk / T::kChunksPerRow, pos = chunk % T::kChunksPerRow;
      const int swz = decltype(is_k)::value ? T::swz_k(row) : T::swz_v(row);
      const uint32_t src = (uint32_t)row * row_bytes + 16u * (uint32_t)(pos ^ swz);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(lds_tile + 512 * (wave * kLoadsPerWave + i)), 16,
                                               (int)src, (int)((uint32_t)j * tile_bytes), 0, 0);
    }
  };

  // Per-lane LDS element offsets of the operand reads (row part + swizzled chunk part).
  // K fragment of MFMA step ks: row r (+32 per key block), chunk 2 ks + hh.  The swizzle only touches the low four
  // bits of the chunk index, so steps 8 apart (d = 256) differ by a constant 16 chunks and share one register.
  constexpr int kKAddrs = kKSteps < 8 ? kKSteps : 8;
  int k_addr[kKAddrs];
#pragma unroll
  for (int ks = 0; ks < kKAddrs; ++ks) k_addr[ks] = r * D + 8 * ((2 * ks + hh) ^ T::swz_k(r));
  int v_addr[kDBlocks];  // V fragment of d-block db: row 4 hh + (lane%16)/4 (+16 per step, +8 for the upper half)
  {
    const int l16 = lane & 15;
    const int row0 = 4 * hh + (l16 >> 2);
#pragma unroll
    for (int db = 0; db < kDBlocks; ++db) {
      const int chunk = 4 * db + 2 * ((lane >> 4) & 1) + ((l16 & 3) >> 1);
      v_addr[db] = row0 * D + 8 * (chunk ^ T::swz_v(row0)) + 4 * (l16 & 1);
    }
  }

  // Accumulators of Algorithm 2: O^T (fp32), the rowmax reference and the running rowsum.  Each half
  // of the wavefront keeps the partial rowsum of its own keys; the two are added in the epilogue.
  f32x16 ot[kDBlocks];
  f32x16 st[kKBlocks];  // S^T of the tile being processed
  float m_ref;          // reference point of the exponentials, in units of the unscaled logits q.k
  float mc_ref;         // m_ref * scale * log2(e)
  float l_run;

  // Operand fragment of MFMA step `step` of GEMM-I (K rows) / GEMM-II (V columns, transposed by the load).
  auto k_frag = [&](const uint16_t* kt, int step) __attribute__((always_inline)) -> u32x4 {
    const int ks = step / kKBlocks, kb = step % kKBlocks;
    return *reinterpret_cast<const u32x4*>(kt + k_addr[ks % kKAddrs] + (ks / kKAddrs) * 128 + kb * 32 * D);
  };
  auto v_frag = [&](const uint16_t* vt, int step) __attribute__((always_inline)) -> u32x4 {
    const int t = step / kDBlocks, db = step % kDBlocks;
    const uint16_t* p = vt + v_addr[db] + t * 16 * D;
    const u32x2 lo = lds_read_tr16(p);
    const u32x2 hi = lds_read_tr16(p + 8 * D);
    return u32x4{lo[0], lo[1], hi[0], hi[1]};
  };

  // GEMM-I (transposed): S^T[key][query] = K_j Q_i^T, fragments prefetched kRing steps ahead.
  auto gemm1 = [&](const uint16_t* kt) __attribute__((always_inline)) {
    u32x4 ring[kRing];
#pragma unroll
    for (int i = 0; i < kRing; ++i) ring[i] = k_frag(kt, i);
#pragma unroll
    for (int kb = 0; kb < kKBlocks; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) st[kb][v] = 0.f;
#pragma unroll
    for (int i = 0; i < kSteps1; ++i) {
      const int ks = i / kKBlocks, kb = i % kKBlocks;
      st[kb] = E::mfma(ring[i % kRing], qf[ks], st[kb]);
      if (i + kRing < kSteps1) ring[i % kRing] = k_frag(kt, i + kRing);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // One iteration of Algorithm 2's inner loop, software-pipelined by one tile on the K side: softmax of
  // S_j, O += P~_j V_j, then S_{j+1} = K_{j+1} Q^T.  Every iteration thus has one block of softmax
  // arithmetic and one block of back-to-back MFMAs, which the two wavefronts sharing a SIMD overlap.
  // kNext: a tile j+1 exists.
  // mask_tag: the tile straddles the causal diagonal; `visible` is then the largest value of
  // 32 kb + 8 (v/4) + v%4 (the key's position in the tile minus this half's 4 hh) that register v of key
  // block kb may have for its key to be at or before this lane's query.
  bool hurry = false;  // kFlagSync: this wavefront did not have to wait at its last boundary, so it is among the slowest
  // kSplitRefill: the K half of the refill, issued inside iteration jj (see stage_ahead there): K tile jj + kNBuf,
  // or, past the end of a chained pass that another one follows, that one's tile
  auto split_k_refill = [&](int jj, uint16_t* k_refill) __attribute__((always_inline)) {
    if (jj + kNBuf < n_tiles) stage_in(true_type{}, k_rsrc, jj + kNBuf, k_refill);
    else if (kChain && more) stage_in(true_type{}, rsrc_of(K, bh_next), jj + kNBuf - n_tiles, k_refill);
  };
  auto iteration = [&](auto next_tag, auto mask_tag, int visible, const uint16_t* v_cur, const uint16_t* k_next,
                       int jj, uint16_t* k_refill) __attribute__((always_inline)) {
    if constexpr (decltype(mask_tag)::value) {
      // S_ij = -inf for j > i: the exponential below turns it into an exact 0 in P~ and in the rowsum.  Key 0
      // is visible to every query, so the reference point is finite from the first tile on.
#pragma unroll
      for (int kb = 0; kb < kKBlocks; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (32 * kb + 8 * (v / 4) + (v % 4) > visible) st[kb][v] = -INFINITY;
    }
    // ---- online softmax for this lane's query (Algorithm 2: rowmax, P~, rowsum, rescale) ----
    // The scale is folded into the exponent, exp(scale*(s - m)) = exp2(s*c - m*c) with c = scale*log2(e), and
    // the maximum is taken on the unscaled logits (valid for scale > 0).
    //
    // The reference point m of the exponentials only has to keep them in range, it need not be the running
    // maximum of Algorithm 2: the result is unchanged because the reference cancels in O / l.  It is moved (and
    // O, l rescaled by exp(m_old - m_new)) only when a tile would otherwise produce a P~ above 2^kLazyLog2.
    if (kFlagSync && hurry) __builtin_amdgcn_s_setprio(2);
    else __builtin_amdgcn_s_setprio(0);
    constexpr bool kMasked = decltype(mask_tag)::value;
    constexpr float kLazyLimit = 256.0f;  // 2^kLazyLog2
    // d = 256 takes the maximum on every tile and skips the rescale when no row of the wavefront moves; the lazy
    // path reaches update_reference only when some row does (or on first and masked tiles)
    constexpr bool kSkipIdleRescale = D == 256;
    static_assert(kLazyLog2 == 8.0f, "kLazyLimit is 2^kLazyLog2");
    u32x4 ring[kRing];   // operand fragments on their way from LDS to the MFMAs
    float rowsum[2];
    u32x4 pf[kTSteps];

    // Row maximum of this tile (both halves of the wavefront), the move of the reference point for the rows that
    // `moves(mx)` selects, and the rescale of l and O.
    auto update_reference = [&](auto moves) __attribute__((always_inline)) {
      // The maxima below are inline assembly, for which the compiler inserts no wait states: S^T may have been
      // written by an MFMA (8 passes) shortly before, so the distance an MFMA result needs before a vector
      // instruction may read it is put here by hand (this path runs on first, masked and rare tiles only).
      asm volatile("s_nop 15\n\ts_nop 3");
      float mx = max2_raw(st[0][0], st[0][1]);
#pragma unroll
      for (int kb = 0; kb < kKBlocks; ++kb)
#pragma unroll
        for (int v = (kb == 0 ? 2 : 0); v < 16; v += 2) mx = max3_raw(mx, st[kb][v], st[kb][v + 1]);
      mx = max_with_partner_half_raw(mx);
      const bool move = moves(mx);
      if (!kSkipIdleRescale || __builtin_amdgcn_ballot_w64(move) != 0) {
        const float m_new = move ? mx : m_ref;
        const float mc_new = m_new * scale_log2e;
        // exp(m_old - m_new); 0 on the first tile.  A row that stays (the branch is taken when any row of the
        // wavefront moves) gets exactly 1, not exp2 of a contracted m*c - m*c that may differ from 0 in the last
        // bit: a row's result must not depend on what the other rows of the wavefront hold.
        const float alpha = move ? __builtin_amdgcn_exp2f(mc_ref - mc_new) : 1.0f;
        m_ref = m_new;
        mc_ref = mc_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) ot[db][v] *= alpha;
      }
    };
    // Issued once per tile, right before its first round of exponentials:
    //  * the second half of the refill (kSplitRefill): K tile jj + kNBuf into the buffer that held K tile jj, which
    //    every wavefront finished reading before the barrier that precedes this iteration.  The V half was issued
    //    right after that barrier.  At d = 256 a tile pair is 16 loads per wavefront; issued as one burst they
    //    overrun the queue between the wavefronts and the texture unit, which accepts about four loads per
    //    wavefront at once and then only as fast as the path into LDS drains, and every wavefront of the workgroup
    //    stands still meanwhile;
    //  * the first V fragments of GEMM-II: independent of P~, so their LDS latency hides behind the exponentials.
    auto stage_ahead = [&]() __attribute__((always_inline)) {
      if constexpr (kSplitRefill) split_k_refill(jj, k_refill);
#pragma unroll
      for (int i = 0; i < kRing; ++i) ring[i] = v_frag(v_cur, i);
    };
    // P~ = exp2(s*c - m*c): the rowsum is taken in fp32 from the unrounded values (Algorithm 2 keeps it in
    // the accumulator type); rounded to 16 bit, registers 8t..8t+7 of a 32-key block are the 8 B-operand
    // slots of MFMA step t.
    auto exponentials = [&]() __attribute__((always_inline)) {
      rowsum[0] = 0.f;
      rowsum[1] = 0.f;
#pragma unroll
      for (int kb = 0; kb < kKBlocks; ++kb) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int v = 8 * t + 2 * c;
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kb][v], scale_log2e, -mc_ref));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kb][v + 1], scale_log2e, -mc_ref));
            rowsum[0] += p0;
            rowsum[1] += p1;
            pf[kb * 2 + t][c] = E::pack2(p0, p1);
          }
        }
      }
    };
    // A row moves when its tile maximum is more than 2^kLazyLog2 above the reference (the first tile's reference is
    // -inf, so every row moves there).
    auto exceeds = [&](float mx) __attribute__((always_inline)) { return (mx - m_ref) * scale_log2e > kLazyLog2; };

    if constexpr (D == 256) {
      // One wavefront per SIMD and every register in use: S cannot stay live across a first round of
      // exponentials, so the row maximum is taken on every tile.
      update_reference(exceeds);
      stage_ahead();
      exponentials();
    } else {
      // A tile first exponentiates against the reference it inherits and looks at the partial row sums: a P~
      // above the limit makes the partial row sum of its lane exceed the limit.  Only then -- and on the first
      // tile (reference -inf) and on tiles with masked entries (S holds -inf) -- does the wavefront take the row
      // maximum, move the reference of the rows concerned and exponentiate again.  Which rows move is decided
      // from the row's own values, never from another row's: on first and masked tiles by the maximum, otherwise
      // by the row's two partial sums.  (Finite inputs and a finite reference: the sums are in [0, +inf].)
      stage_ahead();
      bool need_max = kMasked || jj == 0;   // wavefront-uniform
      float sum_seen = 0.f;
      if (!need_max) {
        exponentials();
        sum_seen = rowsum[0] + rowsum[1];
        need_max = __builtin_amdgcn_ballot_w64(sum_seen > kLazyLimit) != 0;
      }
      if (need_max) {
        update_reference([&](float mx) __attribute__((always_inline)) {
          if (kMasked || jj == 0) return exceeds(mx);
          const uint32_t u = __builtin_bit_cast(uint32_t, sum_seen);
          const auto both = __builtin_amdgcn_permlane32_swap(u, u, false, false);
          return __builtin_bit_cast(float, (uint32_t)both[0]) > kLazyLimit ||
                 __builtin_bit_cast(float, (uint32_t)both[1]) > kLazyLimit;
        });
        exponentials();
      }
    }
    l_run += rowsum[0] + rowsum[1];
    __builtin_amdgcn_sched_barrier(0);

    // ---- GEMM-II (transposed): O^T[d][query] += V_j^T P~^T.  Slot i of lane-half hh in step t is key
    // 16t + 8(i/4) + 4hh + i%4, the key of accumulator register 8t+i of GEMM-I.  GEMM-I of the next tile
    // follows in the same stream of MFMA steps, so its first K fragments are fetched under the last MFMAs of
    // GEMM-II and no LDS latency is exposed between the two products.
    if (kFlagSync && hurry) __builtin_amdgcn_s_setprio(3);
    else __builtin_amdgcn_s_setprio(1);
    constexpr bool kNext = decltype(next_tag)::value;
    constexpr int kStepsAll = kSteps2 + (kNext ? kSteps1 : 0);
    auto any_frag = [&](int step) __attribute__((always_inline)) -> u32x4 {
      return step < kSteps2 ? v_frag(v_cur, step) : k_frag(k_next, step - kSteps2);
    };
#pragma unroll
    for (int i = 0; i < kStepsAll; ++i) {
      if (i < kSteps2) {
        const int t = i / kDBlocks, db = i % kDBlocks;
        ot[db] = E::mfma(ring[i % kRing], pf[t], ot[db]);
      } else {
        const int i1 = i - kSteps2, ks = i1 / kKBlocks, kb = i1 % kKBlocks;
        if (ks == 0) {
          f32x16 zero;
#pragma unroll
          for (int v = 0; v < 16; ++v) zero[v] = 0.f;
          st[kb] = E::mfma(ring[i % kRing], qf[ks], zero);
        } else {
          st[kb] = E::mfma(ring[i % kRing], qf[ks], st[kb]);
        }
      }
      if (i + kRing < kStepsAll) ring[i % kRing] = any_frag(i + kRing);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // LDS schedule.  K tile t lives in k_lds[t % kNBuf], V tile t in v_lds[t % kNBuf].  Iteration j reads
  // V tile j and K tile j+1.  With a barrier per tile (4-wavefront kernels) those two tiles are dead after the
  // barrier that ends the iteration, and their buffers are refilled with K tile j+1+kNBuf and V tile j+kNBuf;
  // the loads needed by iteration j+1 (K tile j+2, V tile j+1) were issued kNBuf-1 barriers earlier; every
  // barrier issues 2*kLoadsPerWave loads per wavefront, so while every barrier issues its full set it is enough
  // to wait until at most (kNBuf-2)*2*kLoadsPerWave loads are outstanding.  Without barriers (kFlagSync) the
  // refill is one tile behind that, see `boundary`.
  constexpr int kRelaxedVmcnt = (kNBuf - 2) * 2 * kLoadsPerWave;
  static_assert(kRelaxedVmcnt < 64, "vmcnt is a 6-bit counter");
  constexpr int kWaitRelaxed = (kRelaxedVmcnt & 15) | ((kRelaxedVmcnt >> 4) << 14) | 0x0F70;
  constexpr int kWaitAll = 0x0F70;  // vmcnt(0), expcnt and lgkmcnt left alone

  uint16_t* const k_buf[4] = {k_lds0, k_lds1, k_lds2, k_lds3};
  uint16_t* const v_buf[4] = {v_lds0, v_lds1, v_lds2, v_lds3};

  // end of iteration j: publish what iteration j+1 reads, then refill the two dead buffers
  auto boundary = [&](auto relaxed_tag, int j, uint16_t* k_fill, uint16_t* v_fill) __attribute__((always_inline)) {
    if constexpr (kFlagSync) {
      // Arrival j of a wavefront says: my reads of V tile j and K tile j+1 are over, and my share of the loads
      // issued at the previous boundary (K tile j+3, V tile j+2) has landed.  A wavefront leaves boundary j when
      // every wavefront has made arrival j-1: then K tile j+2 and V tile j+1, which iteration j+1 reads, are
      // complete, and V tile j-1 and K tile j are dead, so their buffers (k_fill, v_fill) take K tile j+kNBuf and
      // V tile j-1+kNBuf.  A wavefront makes arrival j before it waits for the others' arrival j-1, so it can be two
      // arrivals ahead of the slowest: arrivals are counted per iteration, iteration j in entry j % 4 (entries are
      // reused four iterations later, far beyond that lead), and arrival j-1 is complete when its entry has
      // reached kWv * ((j-1)/4 + 1).  The wait is bounded: a wavefront that gives up poisons its rowsum, so the
      // error shows in O and LSE instead of hanging the GPU.
      // a first look at the others' count, under way while this wavefront waits for its own loads
      // (with chained Q tiles the iterations are counted along the whole stream: n_tiles is a multiple of 4)
      const int g = stream_base + j;
      uint32_t seen = __hip_atomic_load(&arrivals[(j + 3) & 3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      __builtin_amdgcn_s_waitcnt(kWaitAll);
      if (lane == 0) __hip_atomic_fetch_add(&arrivals[j & 3], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
      const uint32_t target = g > 0 ? (uint32_t)(kWv * ((g - 1) / 4 + 1)) : 0u;
      int spins = 0;
      while (seen < target) {
        __builtin_amdgcn_s_sleep(1);
        if (++spins > kSpinLimit) {
          l_run = __builtin_nanf("");
          break;
        }
        seen = __hip_atomic_load(&arrivals[(j + 3) & 3], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");  // the tiles are read only after the count was seen
      hurry = spins == 0;
      const int kt = j + kNBuf, vt = j - 1 + kNBuf;
      if (kt < n_tiles) stage_in(true_type{}, k_rsrc, kt, k_fill);
      else if (more) stage_in(true_type{}, rsrc_of(K, bh_next), kt - n_tiles, k_fill);
      if (vt < n_tiles) stage_in(false_type{}, v_rsrc, vt, v_fill);
      else if (more) stage_in(false_type{}, rsrc_of(V, bh_next), vt - n_tiles, v_fill);
      return;
    }
    if constexpr (decltype(relaxed_tag)::value) __builtin_amdgcn_s_waitcnt(kWaitRelaxed);
    else __builtin_amdgcn_s_waitcnt(kWaitAll);
    __syncthreads();
    // (a chained pass that another one follows goes on with that one's first tiles)
    if constexpr (!kSplitRefill) {
      if (j + 1 + kNBuf < n_tiles) stage_in(true_type{}, k_rsrc, j + 1 + kNBuf, k_fill);
      else if (kChain && more) stage_in(true_type{}, rsrc_of(K, bh_next), j + 1 + kNBuf - n_tiles, k_fill);
    }
    if (j + kNBuf < n_tiles) stage_in(false_type{}, v_rsrc, j + kNBuf, v_fill);
    else if (kChain && more) stage_in(false_type{}, rsrc_of(V, bh_next), j + kNBuf - n_tiles, v_fill);
  };
  // buffers refilled at the boundary after iteration j+i of a group of kNBuf iterations (see `boundary`)
  constexpr int kKFillShift = kFlagSync ? 0 : 1, kVFillShift = kFlagSync ? kNBuf - 1 : 0;

  // Q fragment of Q tile `qtile`: B operand of S^T = K Q^T, straight from global memory into registers
  auto load_q = [&](size_t base, int qtile) __attribute__((always_inline)) {
    const int row = qtile * kRows + wave * 32 + r;
    const int row_ld = kRagged ? min(row, Nq - 1) : row;
    const uint16_t* qp = Q + base + (size_t)row_ld * row_stride + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < kKSteps; ++ks) qf[ks] = *reinterpret_cast<const u32x4*>(qp + 16 * ks);
  };

  // the arrival counters start at zero; the first pass's barrier publishes them
  if (kFlagSync && tid < 4) arrivals[tid] = 0;
  for (int pass = 0; pass < n_pass; ++pass) {
    // causal pair: the first Q tile's last K/V reads are over before the buffers are refilled
    if (pass > 0 && !kChain) __syncthreads();
    if constexpr (kChain) {
      // head and Q tile of pass p: chain step p (causal: p / 2, the heavy tile of the pair first, then the light one)
      auto locate = [&](int p, int& bh_, int& qt_) {
        const int t = tile + (kCausal ? p >> 1 : p) * chain_stride;
        bh_ = t / n_items;
        const int it = t - bh_ * n_items;
        qt_ = kCausal ? ((p & 1) == 0 ? n_qtiles - 1 - it : it) : it;
      };
      locate(pass, bh, qt);
      head_base = q_base_of(bh);
      k_rsrc = rsrc_of(K, bh);
      v_rsrc = rsrc_of(V, bh);
      more = pass + 1 < n_pass;
      if (more) locate(pass + 1, bh_next, qt_next);
    } else {
      qt = kCausal ? (pass == 0 ? n_qtiles - 1 - item : item) : item;
    }
    q_row = qt * kRows + wave * 32 + r;
    // a multiple of kNBuf in every case; causal: the keys up to the end of this Q tile
    n_tiles = kCausal ? (qt + 1) * kNBuf : kRagged ? (Nk + kNBuf * kBc - 1) / (kNBuf * kBc) * kNBuf : Nk / kBc;
#pragma unroll
    for (int db = 0; db < kDBlocks; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) ot[db][v] = 0.f;
    m_ref = -INFINITY;
    mc_ref = -INFINITY;
    l_run = 0.f;

    // A chained Q tile after the first finds its ring filled, its Q fragment loaded and its first S computed by
    // the end of the pass before it.
    if (!kChain || pass == 0) {
      load_q(head_base, qt);
      static_for<kNBuf>([&](auto t) { stage_in(true_type{}, k_rsrc, decltype(t)::value, k_buf[decltype(t)::value]); });
      static_for<kNBuf - 1>([&](auto t) { stage_in(false_type{}, v_rsrc, decltype(t)::value, v_buf[decltype(t)::value]); });
      // The Q fragment must have landed before the loop so that no wait for it is placed inside the loop.
#pragma unroll
      for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(qf[ks]));
      __builtin_amdgcn_s_waitcnt(kWaitAll);
      __syncthreads();
      gemm1(k_lds0);
      __syncthreads();  // every wavefront has finished reading K tile 0 before its buffer is refilled
      if constexpr (!kFlagSync) {   // (with kFlagSync the first boundary issues these two)
        if constexpr (!kSplitRefill) {
          if (kNBuf < n_tiles) stage_in(true_type{}, k_rsrc, kNBuf, k_lds0);
        }
        if (kNBuf - 1 < n_tiles) stage_in(false_type{}, v_rsrc, kNBuf - 1, v_buf[kNBuf - 1]);
      }
    }

    // partial tiles: wavefronts whose rows all lie past the last query keep the boundaries and skip the arithmetic
    // (not in the two partial-tile kernels that have no register left for one more condition)
    constexpr bool kSkipDeadRows = kRagged && D <= 128 && !(D == 128 && kCausal);
    const bool rows_live = !kSkipDeadRows || qt * kRows + wave * 32 < Nq;   // wavefront-uniform
    int j = 0;
    for (; j + kNBuf < n_tiles; j += kNBuf) {  // every barrier of these iterations issues its full set of loads
      static_for<kNBuf>([&](auto t) {
        constexpr int i = decltype(t)::value;
        if (rows_live) iteration(true_type{}, false_type{}, 0, v_buf[i], k_buf[(i + 1) % kNBuf], j + i, k_buf[i]);
        boundary(true_type{}, j + i, k_buf[(i + kKFillShift) % kNBuf], v_buf[(i + kVFillShift) % kNBuf]);
      });
    }
    // last kNBuf tiles: wait for everything, and the very last tile has no successor.  Under the causal mask
    // these are exactly the tiles of this Q tile's own rows, the ones the diagonal crosses.
    // Without the causal mask the same tiles are the only ones that can hold keys past Nk-1.
    using mask_tail = std::integral_constant<bool, kCausal || kRagged>;
    static_for<kNBuf>([&](auto t) {
      constexpr int i = decltype(t)::value;
      // causal: (q_row - first key of tile j+i) - 4 hh; a stored row (q_row < Nq = Nk) never sees a key past
      // Nk-1 through it.  Otherwise: (last key - first key of tile j+i) - 4 hh.
      int visible = kCausal ? wave * 32 + r - 4 * hh - i * kBc : Nk - 1 - (j + i) * kBc - 4 * hh;
      // computed here, not hoisted above the main loop where 32 comparison results per tile would sit in
      // scalar registers for the whole loop
      if constexpr (mask_tail::value) asm volatile("" : "+v"(visible));
      // Under the causal mask a tile of the Q tile's own rows lies wholly above the diagonal for the wavefronts whose
      // 32 rows come before its first key: for them it would contribute exact zeros, so they leave its arithmetic
      // out (and keep every boundary: the others still count on their loads and arrivals).  The same goes, for every
      // wavefront, for a padding tile that only rounds the tile count up and holds no key at all.
      // And a wavefront whose 32 rows all lie past the last query (partial last Q tile) computes nothing at all.
      const bool live = (!kCausal || i * kBc <= wave * 32 + 31) && (!kRagged || (j + i) * kBc < Nk) && rows_live;
      if constexpr (i + 1 < kNBuf) {
        if (live) iteration(true_type{}, mask_tail{}, visible, v_buf[i], k_buf[(i + 1) % kNBuf], j + i, k_buf[i]);
        else if constexpr (kSplitRefill) split_k_refill(j + i, k_buf[i]);   // its loads are still this wavefront's
        boundary(false_type{}, j + i, k_buf[(i + kKFillShift) % kNBuf], v_buf[(i + kVFillShift) % kNBuf]);
      } else {
        // Q is last used by the GEMM-I of the iteration before this one: the next Q tile's fragment is fetched
        // under this iteration
        if (kChain && more) load_q(q_base_of(bh_next), qt_next);
        if (live) iteration(false_type{}, mask_tail{}, visible, v_buf[i], k_buf[(i + 1) % kNBuf], j + i, k_buf[i]);
        else if constexpr (kSplitRefill) split_k_refill(j + i, k_buf[i]);
        if (kChain && more) {
          // S of the next Q tile's first K/V tile (stream tile n_tiles, complete since the boundary two iterations
          // ago), then the boundary that every iteration of the stream ends with.  O, l and the reference of this
          // Q tile are untouched by both and are written out below.
#pragma unroll
          for (int ks = 0; ks < kKSteps; ++ks) asm volatile("" : "+v"(qf[ks]));
          gemm1(k_buf[(i + 1) % kNBuf]);
          boundary(false_type{}, j + i, k_buf[(i + kKFillShift) % kNBuf], v_buf[(i + kVFillShift) % kNBuf]);
        }
      }
    });

    // Epilogue: O_i = O_i / rowsum, LSE_i = m_i + ln(rowsum) (natural log, scaled logits).
    const float l_tot = sum_with_partner_half(l_run);
    const float inv_l = 1.0f / l_tot;
    if (kRowStores || !kRagged || q_row < Nq) {   // (row stores: every lane takes part, rows are checked one by one)
      if constexpr (kRowStores) {
        // Each 32-column block goes through the wavefront's own LDS slab (row r at
        // byte 64 r, its four 16-byte chunks XOR-permuted by (r / 4) % 4 against bank conflicts) and leaves as
        // two stores of 16 rows x 64 bytes.  Only this wavefront touches its slab, and LDS executes a wavefront's
        // accesses in order, so no barrier is involved.
        uint16_t* slab = o_slab + wave * 1024;
        const int rrow = lane >> 2, rchunk = lane & 3;   // as a reader: row (+16 for the second half), chunk
        uint16_t* orow = O + head_base + (size_t)(qt * kRows + wave * 32 + rrow) * row_stride + 8 * rchunk;
#pragma unroll
        for (int db = 0; db < kDBlocks; ++db) {
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            // accumulator registers 4g..4g+3 hold d = 32 db + 8 g + 4 hh + (0..3) of this lane's query
            u32x2 w = {E::pack2(ot[db][4 * g + 0] * inv_l, ot[db][4 * g + 1] * inv_l),
                       E::pack2(ot[db][4 * g + 2] * inv_l, ot[db][4 * g + 3] * inv_l)};
            *reinterpret_cast<u32x2*>(slab + r * 32 + 8 * (g ^ ((r >> 2) & 3)) + 4 * hh) = w;
          }
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            const int row = rrow + 16 * half;
            const u32x4 piece = *reinterpret_cast<const u32x4*>(slab + row * 32 + 8 * (rchunk ^ ((row >> 2) & 3)));
            if (!kRagged || qt * kRows + wave * 32 + row < Nq)
              *reinterpret_cast<u32x4*>(orow + (size_t)(16 * half) * row_stride + 32 * db) = piece;
          }
        }
      } else {
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
      }
      if (LSE != nullptr && hh == 0 && (!kRagged || q_row < Nq)) {
        LSE[(size_t)bh * Nq + q_row] = mc_ref * 0.69314718055994530942f + __builtin_logf(l_tot);
      }
    }
    if constexpr (kChain) stream_base += n_tiles;  // every pass's tile count is a multiple of kNBuf
  }  // pass
}

constexpr int kRows256 = 256;  // query rows per workgroup of the 8-wavefront shape

// Enqueues `kernel` and reports this launch's own status (not whatever error an earlier, unrelated HIP call left).
template <class... Params, class... Args>
int enqueue(void (*kernel)(Params...), int grid, int block, hipStream_t stream, Args... args) {
  std::tuple<Params...> values{static_cast<Params>(args)...};
  void* ptrs[sizeof...(Params)];
  std::apply([&](auto&... v) { int i = 0; ((ptrs[i++] = &v), ...); }, values);
  const hipError_t err = hipLaunchKernel(reinterpret_cast<const void*>(kernel), dim3((unsigned)grid), dim3((unsigned)block),
                                         ptrs, 0, stream);
  return err == hipSuccess ? FA2_OK : FA2_ERR_LAUNCH;
}

// One instantiation of the 32-row kernel.
template <int DT, int D, int kWv, int kNBuf, bool kCausal, bool kRagged>
int launch_rows32(const void* Q, const void* K, const void* V, void* O, float* LSE, int H, int Nq, int Nk,
                  float scale_log2e, int n_qtiles, int total, hipStream_t stream, int chain = 1) {
  return enqueue(fa2_fwd_kernel<DT, D, kWv, kNBuf, kCausal, kRagged>, total, kWv * 64, stream,
                 static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K), static_cast<const uint16_t*>(V),
                 static_cast<uint16_t*>(O), LSE, H, Nq, Nk, scale_log2e, n_qtiles, total, chain);
}


template <int DT, int D>
int launch(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int Nq, int Nk, float scale,
           int variant, int mask, hipStream_t stream) {
  const float scale_log2e = scale * 1.44269504088896340736f;
  const bool rows256 = variant == FA2_VARIANT_NARROW8;
  const bool causal = mask == FA2_MASK_CAUSAL;
  const bool ragged = Nq % kBr != 0 || Nk % kBr != 0;  // 128-row shape only (checked by the caller)
  const int rows = rows256 ? kRows256 : kBr;
  const int n_qtiles = (Nq + rows - 1) / rows;
  // causal: one workgroup per pair of Q tiles (n_qtiles-1-p, p)
  const long long total_ll = (long long)B * H * (causal ? (n_qtiles + 1) / 2 : n_qtiles);
  if (total_ll > 0x7fffffffLL) return FA2_ERR_UNSUPPORTED;
  const int total = (int)total_ll;
  if (rows256) {  // exact tiles, d <= 128 (checked by the caller)
    if constexpr (D <= 128) {
      // When the Q tiles (causal: the pairs of Q tiles, all complete) fill whole rounds of the CUs, one workgroup
      // per CU takes a Q tile (pair) of every round.
      const int chain = total % kCUs == 0 && !(causal && n_qtiles % 2 != 0) ? total / kCUs : 1;
      if (causal)
        return launch_rows32<DT, D, 8, 4, true, false>(Q, K, V, O, LSE, H, Nq, Nk, scale_log2e, n_qtiles, total / chain,
                                                       stream, chain);
      return launch_rows32<DT, D, 8, 4, false, false>(Q, K, V, O, LSE, H, Nq, Nk, scale_log2e, n_qtiles, total / chain,
                                                      stream, chain);
    } else {
      return FA2_ERR_UNSUPPORTED;
    }
  } else if (causal) {
    if (ragged) return launch_rows32<DT, D, 4, 2, true, true>(Q, K, V, O, LSE, H, Nq, Nk, scale_log2e, n_qtiles, total, stream);
    // d = 256: pairs chained like the Q tiles of the unmasked case (whole rounds of complete pairs)
    const int chain = D == 256 && total % kCUs == 0 && n_qtiles % 2 == 0 ? total / kCUs : 1;
    return launch_rows32<DT, D, 4, 2, true, false>(Q, K, V, O, LSE, H, Nq, Nk, scale_log2e, n_qtiles, total / chain, stream,
                                                   chain);
  }
  if (ragged) return launch_rows32<DT, D, 4, 2, false, true>(Q, K, V, O, LSE, H, Nq, Nk, scale_log2e, n_qtiles, total, stream);
  // d = 256 (one workgroup per CU): when the Q tiles fill whole rounds of the CUs, one workgroup per CU takes a Q tile
  // of every round, as in the 256-row shape
  const int chain = D == 256 && total % kCUs == 0 ? total / kCUs : 1;
  return launch_rows32<DT, D, 4, 2, false, false>(Q, K, V, O, LSE, H, Nq, Nk, scale_log2e, n_qtiles, total / chain, stream,
                                                  chain);
}

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// The tile shape that FA2_VARIANT_AUTO stands for (sizes already validated by the caller).
int choose_variant(int B, int H, int Nq, int Nk, int d, int mask) {
  // Measured on MI355X with N(0,1) inputs: when its Q tiles fill whole rounds of the chip's 256 CUs (one workgroup
  // per CU, which then takes one Q tile of every round), the 8-wavefront, 256-row shape is faster than the
  // 4-wavefront, 128-row shape by 3-6 % at d = 128 at every N, and by 1-2 % at d = 64 from N = 4096 on (at d = 64
  // below N = 2048 its two wavefronts per SIMD against three lose 2-5 %).  With many rounds that are not whole it
  // still gains at d = 128 from N = 2048 on; with few, the 128-row shape, two workgroups per CU, spreads the
  // remainder better.  d = 256 and partial tiles exist in the 128-row shape only.
  // Under the causal mask (one workgroup per pair of Q tiles, no chaining) it gains 1-3 % at d = 128 from N = 2048 on.
  const bool causal = mask == FA2_MASK_CAUSAL;
  const long long qt256 = Nq / kRows256;
  const long long wg256 = (long long)B * H * (causal ? (qt256 + 1) / 2 : qt256);
  const bool whole_rounds = wg256 % kCUs == 0;   // unmasked: then one workgroup per CU chains a Q tile of every round
  const bool rows256 = d <= 128 && Nq == Nk && Nq % kRows256 == 0 &&
                       (causal ? d == 128 && Nq >= 2048 && (whole_rounds || wg256 >= 16 * kCUs)
                               : (whole_rounds && (d == 128 || Nq >= 2048)) ||
                                     (d == 128 && wg256 >= 16 * kCUs && Nq >= 2048));
  return rows256 ? FA2_VARIANT_NARROW8 : FA2_VARIANT_NARROW;
}

int run(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int Nq, int Nk, int d,
        float scale, int dtype, int variant, int mask, void* stream) {
  // All validation happens before the first HIP call: an error launches nothing.
  if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr) return FA2_ERR_INVALID_ARG;
  if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || d <= 0) return FA2_ERR_INVALID_ARG;
  if (!(scale > 0.0f) || !(scale <= 3.0e38f)) return FA2_ERR_INVALID_ARG;  // rejects NaN, inf, <= 0
  if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) || !aligned(LSE, 4))
    return FA2_ERR_INVALID_ARG;
  if (variant != FA2_VARIANT_AUTO && variant != FA2_VARIANT_NARROW && variant != FA2_VARIANT_NARROW8)
    return FA2_ERR_INVALID_ARG;
  if (mask != FA2_MASK_NONE && mask != FA2_MASK_CAUSAL) return FA2_ERR_INVALID_ARG;
  if (dtype != FA2_FP16 && dtype != FA2_BF16) return FA2_ERR_UNSUPPORTED;
  if (d != 64 && d != 128 && d != 256) return FA2_ERR_UNSUPPORTED;
  if (mask == FA2_MASK_CAUSAL && Nq != Nk) return FA2_ERR_UNSUPPORTED;  // the diagonal is defined for a square S only
  // element offsets are computed in 64 bits; the row index b*N+n must still fit the tile arithmetic
  const int n_max = Nq > Nk ? Nq : Nk;
  if ((long long)B * n_max > 0x7fffffffLL) return FA2_ERR_UNSUPPORTED;
  // the K/V rows of one batch entry are addressed with 32-bit byte offsets from a buffer descriptor
  if ((unsigned long long)n_max * (unsigned long long)H * (unsigned long long)d * 2ull >= (1ull << 32))
    return FA2_ERR_UNSUPPORTED;
  if (variant == FA2_VARIANT_AUTO) variant = choose_variant(B, H, Nq, Nk, d, mask);
  if (variant != FA2_VARIANT_NARROW) {
    // the 256-row shape: whole tiles, square, d <= 128
    if (Nq != Nk || Nq % kRows256 != 0 || d == 256) return FA2_ERR_UNSUPPORTED;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == FA2_FP16) {
    return d == 64    ? launch<FA2_FP16, 64>(Q, K, V, O, LSE, B, H, Nq, Nk, scale, variant, mask, s)
           : d == 128 ? launch<FA2_FP16, 128>(Q, K, V, O, LSE, B, H, Nq, Nk, scale, variant, mask, s)
                      : launch<FA2_FP16, 256>(Q, K, V, O, LSE, B, H, Nq, Nk, scale, variant, mask, s);
  }
  return d == 64    ? launch<FA2_BF16, 64>(Q, K, V, O, LSE, B, H, Nq, Nk, scale, variant, mask, s)
         : d == 128 ? launch<FA2_BF16, 128>(Q, K, V, O, LSE, B, H, Nq, Nk, scale, variant, mask, s)
                    : launch<FA2_BF16, 256>(Q, K, V, O, LSE, B, H, Nq, Nk, scale, variant, mask, s);
}

}  // namespace

extern "C" int fa2_fwd_variant(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int N,
                               int d, float scale, int dtype, int variant, void* stream) {
  return run(Q, K, V, O, LSE, B, H, N, N, d, scale, dtype, variant, FA2_MASK_NONE, stream);
}

extern "C" int fa2_fwd_masked(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int N,
                              int d, float scale, int dtype, int mask, void* stream) {
  return run(Q, K, V, O, LSE, B, H, N, N, d, scale, dtype, FA2_VARIANT_AUTO, mask, stream);
}

extern "C" int fa2_fwd_qk(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int Nq,
                          int Nk, int d, float scale, int dtype, int mask, void* stream) {
  return run(Q, K, V, O, LSE, B, H, Nq, Nk, d, scale, dtype, FA2_VARIANT_AUTO, mask, stream);
}

extern "C" int fa2_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H, int N, int d,
                       float scale, int dtype, void* stream) {
  return run(Q, K, V, O, LSE, B, H, N, N, d, scale, dtype, FA2_VARIANT_AUTO, FA2_MASK_NONE, stream);
}

extern "C" int fa2_tile_shape(int B, int H, int Nq, int Nk, int d, int mask) {
  if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0) return FA2_ERR_INVALID_ARG;
  if (mask != FA2_MASK_NONE && mask != FA2_MASK_CAUSAL) return FA2_ERR_INVALID_ARG;
  if (d != 64 && d != 128 && d != 256) return FA2_ERR_UNSUPPORTED;
  if (mask == FA2_MASK_CAUSAL && Nq != Nk) return FA2_ERR_UNSUPPORTED;
  return choose_variant(B, H, Nq, Nk, d, mask);
}

extern "C" const char* fa2_strerror(int code) {
  switch (code) {
    case FA2_OK: return "success";
    case FA2_ERR_INVALID_ARG: return "invalid argument (NULL or misaligned pointer, non-positive size, scale not finite and > 0, or unknown variant or mask)";
    case FA2_ERR_UNSUPPORTED: return "unsupported problem (d must be 64, 128 or 256; dtype fp16 or bf16; the causal mask needs Nq == Nk; the 256-row tile shape needs d <= 128 and N a multiple of 256; sizes must fit 32-bit offsets)";
    case FA2_ERR_LAUNCH: return "the HIP runtime refused the kernel launch";
    default: return "unknown fa2 error code";
  }
}

extern "C" int fa2_version(void) { return 500; /* 0.5.0 */ }
