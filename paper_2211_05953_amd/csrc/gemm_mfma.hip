// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_16x16x32_bf16), fp32 accumulate.
//
// One workgroup computes a BM x BN tile of C, stepping BK = 64 along K.  Each step's A and
// B tiles are copied global -> registers -> LDS (16-byte buffer loads, double-buffered LDS, the
// loads of tile kt+2 in flight during the MFMAs of tile kt).  Operands whose
// global layout is K-contiguous sit in LDS as [row][BK] with the 16-byte chunk index
// XOR-swizzled by row bits (conflict-free ds_read_b128 of MFMA fragments on the 64-bank LDS).  Operands whose
// global layout has K as the slow dimension (B of the forward product, both operands of
// the weight-gradient product) sit in LDS as [BK][cols + pad] and are read through the
// LDS transpose load (ds_read_b64_tr_b16), which hands every lane four consecutive k of
// its own column: no transposed copy of any tensor is ever made in HBM.
//
// Wave w of the workgroup owns a (BM / WM) x (BN / WN) sub-tile as MI x NI MFMA tiles of
// 16 x 16 (k = 32 per instruction).  Operand fragment of one MFMA: lane l holds the 8 consecutive
// k from 8 * (l / 16) of row (A) or column (B) l % 16.  Accumulator layout: lane l, register r holds
// row (l / 16) * 4 + r, column l % 16.  The 16 x 16 x 32 form is used because the step runs at the
// socket power limit: in a register-only loop on random operands it sustains 2.00 PFLOP/s where
// the 32 x 32 x 16 form sustains 1.81 (both reach 2.48 on zeros).
#include <atomic>
#include <type_traits>

#include "common.h"
#include "epilogue.h"

namespace bf {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int BK = 64;
// measured throughput of a compute unit on the smaller tiles relative to the 256 x 256 tile
constexpr double TILE_RATE_MID = 0.84, TILE_RATE_SMALL = 0.68, TILE_RATE_WIDE = 0.95;
constexpr int TPAD = 32;  // padding (elements) of a transposed LDS row: stride = 64 bytes mod 128

template <int BM_, int BN_, int WM_, int WN_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int NT = WM * WN * 64;
  static constexpr int TM = BM / WM, TN = BN / WN;
  static constexpr int MI = TM / 16, NI = TN / 16;
  static_assert(MI % 2 == 0, "the A fragments of a k-step are fetched in two halves");
};

// XOR key of a K-contiguous LDS row (128 bytes = 8 chunks of 16 bytes).  The LDS has 64 banks of 4
// bytes and serves a 16-byte-per-lane read 16 lanes at a time, but not 16 consecutive lanes: the
// first cycle of a 32-lane half takes lanes 0-3, 12-15, 20-23, 24-27, the second the other four
// quads (the bank-conflict counter reads zero for layouts that are conflict-free under this
// grouping and a steady two-way conflict for one that is only conflict-free for consecutive lanes).
// A fragment read has lane l at row l % 16 and logical chunk c + l / 16, so one cycle sees the row
// pairs {0,1}, {2,3}, {12,13}, {14,15} at chunk c and {4,5}, {6,7}, {8,9}, {10,11} at chunk c ^ 1 (or the
// reverse).  The key sends the first four pairs to 0..3 and the others to 4..7: both sets are closed
// under ^ 1, so the 16 (row parity, chunk) slots of a cycle are distinct.
__device__ __forceinline__ int kswz(int row) {
  return ((row >> 1) & 1) | (((row >> 3) & 1) << 1) | ((((row >> 2) ^ (row >> 3)) & 1) << 2);
}

// XOR key (in 16-byte chunks) of a transposed LDS row: rows k and k + 8 are read together by the two
// 16-lane groups of a 32-lane half of the transpose load and sit a multiple of 256 bytes apart;
// moving one of them by 16 columns (32 bytes) puts the two groups on disjoint banks.
__device__ __forceinline__ int tkey(int krow) { return ((krow >> 3) & 1) << 1; }

// bytes of one LDS stage of an operand tile with R rows (m or n extent)
template <bool KCONTIG, int R>
constexpr int stage_elems() { return KCONTIG ? R * BK : BK * (R + TPAD); }

// ---- global -> registers: the thread's 16-byte chunks of an operand tile.  Chunk i of a thread
// sits a fixed number of tile rows below chunk 0, so one per-thread byte offset (global) and one
// per-thread element offset (LDS) serve all chunks: every load is "wave-uniform base (scalar
// registers, moved per k-tile and per chunk) + 32-bit lane offset", every LDS store "lane offset
// + immediate".
template <bool KCONTIG, int R, int NT, bool EVEN = KCONTIG || NT % (R / 8) == 0>
struct Stager {
  static constexpr int CHUNKS = R * BK / 8 / NT;
  static constexpr int ROWSTEP = KCONTIG ? NT / 8 : NT / (R / 8);  // tile rows between a thread's chunks
  static_assert(ROWSTEP % 16 == 0, "the swizzle keys must repeat from chunk to chunk");
  u32x4 v[CHUNKS];
  uint32_t goff;  // byte offset of chunk 0 from the tile's first element
  int loff;       // element offset of chunk 0 inside the LDS tile

  __device__ __forceinline__ void init(size_t ld, int tid) {
    if (KCONTIG) {
      const int row = tid >> 3, kc = tid & 7;  // 8 chunks per row of BK = 64
      goff = (uint32_t)(((size_t)row * ld + kc * 8) * sizeof(bf16_t));
      loff = row * BK + ((kc ^ kswz(row)) << 3);
    } else {
      const int krow = tid / (R / 8), rc = tid % (R / 8);
      goff = (uint32_t)(((size_t)krow * ld + rc * 8) * sizeof(bf16_t));
      loff = krow * (R + TPAD) + ((rc ^ tkey(krow)) << 3);
    }
  }
  // g: operand base (uniform); r0: first row/col of the tile; k0: first k.  Buffer loads: the
  // descriptor carries the tile's base address, the lane offset is a VGPR, the chunk step an SGPR.
  __device__ __forceinline__ void load(const bf16_t* __restrict__ g, size_t ld, int r0, int k0) {
    const bf16_t* base = KCONTIG ? g + (size_t)r0 * ld + k0 : g + (size_t)k0 * ld + r0;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, 0x7fffffff, 0x00020000);
    const int step = (int)((size_t)ROWSTEP * ld * sizeof(bf16_t));
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff, i * step, 0);
  }
  __device__ __forceinline__ void store(bf16_t* lds) const {
    constexpr int LSTEP = KCONTIG ? ROWSTEP * BK : ROWSTEP * (R + TPAD);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) *reinterpret_cast<u32x4*>(lds + loff + i * LSTEP) = v[i];
  }
};

// A transposed tile whose rows (R / 8 chunks) the workgroup's threads do not divide into whole passes (192 columns:
// 24 chunks per k-row, 512 threads): the tile's chunks are dealt out in their linear order, chunk tid + i * NT to
// thread tid, and a thread keeps one global and one LDS offset per chunk (they sit in different rows and columns).
template <int R, int NT>
struct Stager<false, R, NT, false> {
  static constexpr int CPR = R / 8;  // chunks per k-row
  static constexpr int CHUNKS = BK * CPR / NT;
  static_assert(BK * CPR % NT == 0, "the tile's chunks must divide among the threads");
  u32x4 v[CHUNKS];
  uint32_t goff[CHUNKS];
  int loff[CHUNKS];

  __device__ __forceinline__ void init(size_t ld, int tid) {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int c = tid + i * NT, krow = c / CPR, rc = c % CPR;
      goff[i] = (uint32_t)(((size_t)krow * ld + rc * 8) * sizeof(bf16_t));
      loff[i] = krow * (R + TPAD) + ((rc ^ tkey(krow)) << 3);
    }
  }
  __device__ __forceinline__ void load(const bf16_t* __restrict__ g, size_t ld, int r0, int k0) {
    const bf16_t* base = g + (size_t)k0 * ld + r0;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, 0x7fffffff, 0x00020000);
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[i], 0, 0);
  }
  __device__ __forceinline__ void store(bf16_t* lds) const {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) *reinterpret_cast<u32x4*>(lds + loff[i]) = v[i];
  }
};

// Lane part of a K-contiguous fragment address, per k-step: the XOR key only has row bits 1-3, which
// come from the lane (fragments start at multiples of 16 rows), so a fragment's address is this
// offset plus a compile-time multiple of 16 rows and every read takes an immediate.
struct KFragLane {
  int o[2];
  __device__ __forceinline__ void init(int lane) {
    const int l15 = lane & 15;
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) o[kk] = l15 * BK + (((kk * 4 + (lane >> 4)) ^ kswz(l15)) << 3);
  }
};

// The same for a transposed tile of R columns.  The key (16 columns) depends on the lane's 16-lane
// group only; XORed into the column it moves a fragment that starts at an even multiple of 16
// columns up and one that starts at an odd multiple down, hence one offset per parity.
template <int R>
struct TFragLane {
  int o[2];
  __device__ __forceinline__ void init(int lane) {
    const int t = lane & 15, blk = lane >> 4;
    const int k = 8 * blk + (t >> 2), c4 = 4 * (t & 3);
#pragma unroll
    for (int par = 0; par < 2; ++par) o[par] = k * (R + TPAD) + (((16 * par + c4) ^ (tkey(k) << 3)) - 16 * par);
  }
};

// ---- LDS -> MFMA fragment: 8 consecutive k of row/column (r16 + lane % 16), k-step kk (32 wide)
// r16: first row / column of the fragment relative to lds, a multiple of 16 (lds itself starts at a
// multiple of 32 rows / columns of the tile)
template <bool KCONTIG, int R>
__device__ __forceinline__ bf16x8 load_frag(const bf16_t* lds, int r16, int kk, const KFragLane& kl, const TFragLane<R>& tl) {
  if (KCONTIG) {
    return *reinterpret_cast<const bf16x8*>(lds + r16 * BK + kl.o[kk]);
  } else {
    // one transpose load: the 16 lanes of a group read 4 k-rows x 16 columns, 4 columns each, and
    // every lane receives the 4 k of its own column; two of them give the lane its 8 k
    const bf16_t* p = lds + kk * 32 * (R + TPAD) + r16 + tl.o[(r16 >> 4) & 1];
    typedef s16x4 __attribute__((address_space(3))) * lds_v4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p + 4 * (R + TPAD)));  // k + 4: same key
    typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
  }
}

// AK: A is K-contiguous in memory (forward, dgrad); BKC: B is K-contiguous (dgrad)
// SEG_POW2: the k-tiles per segment are a power of two (weight gradient only; true for every
// sequence length that is one): the segment of a k-tile is then a shift, not a division, which
// takes 40 scalar instructions out of the loop (0.7-1 % of the product)
template <typename TL, bool AK, bool BKC, int EPI, typename TO, bool SEG_POW2>
__global__ __launch_bounds__(TL::NT) void gemm_mfma_kernel(int M, int N, int K, const bf16_t* __restrict__ A,
                                                           const bf16_t* __restrict__ B, TO* __restrict__ C,
                                                           const float* __restrict__ bias, const TO* __restrict__ R,
                                                           TO* __restrict__ C2, int accumulate, int tiles_m, int remap,
                                                           int n_seg, size_t seg_a, size_t seg_b, float* __restrict__ colpart,
                                                           int ldk) {
  constexpr int BM = TL::BM, BN = TL::BN, NT = TL::NT, MI = TL::MI, NI = TL::NI;
  constexpr int A_ST = stage_elems<AK, BM>(), B_ST = stage_elems<BKC, BN>();
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
  constexpr int STAGE = A_ST + B_ST;  // stage s: A tile at smem + s * STAGE, B tile right after it

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int wm = w % TL::WM, wn = w / TL::WM;
  // Workgroups go to the 8 XCDs round-robin and each XCD has its own L2: give XCD x a contiguous
  // range of the tile order, and walk that order in groups of 8 row-tiles so that the ~32
  // workgroups an XCD runs at a time form an 8 x 4 block sharing A row-panels and B column-panels.
  int lin = blockIdx.x;
  if (remap) {
    const int per_xcd = gridDim.x >> 3;
    lin = (lin & 7) * per_xcd + (lin >> 3);
  }
  const int tiles_n = gridDim.x / tiles_m;
  const int in_group = 8 * tiles_n;
  int bm, bn;
  if (remap && tiles_m % 8 == 0) {
    const int gi = lin / in_group, rem = lin % in_group;
    bm = gi * 8 + (rem & 7);
    bn = rem >> 3;
  } else {
    bm = lin % tiles_m;
    bn = lin / tiles_m;
  }
  const int m0 = bm * BM, n0 = bn * BN;
  // ldk: row length of the operands that are stored K-contiguous; equal to K except in a split-K launch, where K is
  // the length of the slice this workgroup contracts over
  const size_t lda = AK ? (size_t)ldk : (size_t)M;   // A stored [M,K] or [K,M]
  const size_t ldb = BKC ? (size_t)ldk : (size_t)N;  // B stored [N,K] or [K,N]
  if constexpr (EPI == E_ACCUM && AK) {
    // Split-K launch of a forward / dgrad product (grid.y slices of K): slice y starts K elements further along the
    // contraction and leaves its fp32 partial result in plane y of C ([slices][M][N]); a second kernel adds the
    // planes in order and applies the epilogue.
    const size_t y = blockIdx.y;
    A += y * (size_t)K;
    B += y * (BKC ? (size_t)K : (size_t)K * N);
    C += y * (size_t)M * N;
  }

  f32x4 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
  if constexpr (EPI == E_ACCUM) {
    // Accumulating into the main-grad: the accumulators START from the stored values, so the reads
    // of C overlap the first k-tiles and the epilogue is a plain store (read-modify-write at the end
    // would stall every workgroup of the round on HBM latency at once).
    if (accumulate) {
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const size_t row = m0 + wm * TL::TM + i * 16 + (lane >> 4) * 4 + r;
            const size_t col = n0 + wn * TL::TN + j * 16 + (lane & 15);
            acc[i][j][r] = C[row * (size_t)N + col];
          }
    }
  }

  Stager<AK, BM, NT> sa;
  Stager<BKC, BN, NT> sb;
  sa.init(lda, tid);
  sb.init(ldb, tid);
  // Residual / pre-activation values the epilogue needs (E_BIAS_RES, E_GELU_BWD): the first half is
  // requested before the last k-tile, when the staging registers are free, so that its HBM latency
  // hides behind that tile's MFMAs instead of stalling every workgroup of the round at once; the
  // second half follows after the main loop, when the fragment registers are free, and arrives
  // while the first passes of the epilogue run.
  constexpr int PR = 64, NQ = PR * BN / 8 / NT;
  constexpr bool HAS_R = EPI == E_BIAS_RES || EPI == E_GELU_BWD;
  bf16x8 rpre[HAS_R ? BM / PR : 1][HAS_R ? NQ : 1];
  auto prefetch_r = [&](auto first_half) {
    if constexpr (HAS_R) {
      constexpr int P0 = decltype(first_half)::value ? 0 : BM / PR / 2, P1 = decltype(first_half)::value ? BM / PR / 2 : BM / PR;
#pragma unroll
      for (int p = P0; p < P1; ++p)
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
          const int c = tid + q * NT, lr = c / (BN / 8), lc = (c % (BN / 8)) * 8;
          rpre[p][q] = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const bf16_t*>(R) + (size_t)(m0 + p * PR + lr) * N + n0 + lc);
        }
    }
  };
  const int nk_seg = K / BK, nk = nk_seg * n_seg;
  // k-tile kt lives in segment kt / nk_seg (one segment unless this is a multi-micro-batch weight gradient)
  // (only the weight-gradient product is launched with segments: the others skip the division)
  constexpr bool SEGS = EPI == E_ACCUM;
  const int seg_shift = __builtin_ctz(nk_seg);
  auto seg_of = [&](int kt) { return SEG_POW2 ? kt >> seg_shift : kt / nk_seg; };
  auto seg_a_of = [&](int kt) { return SEGS ? A + (size_t)seg_of(kt) * seg_a : A; };
  auto seg_b_of = [&](int kt) { return SEGS ? B + (size_t)seg_of(kt) * seg_b : B; };
  auto k0_of = [&](int kt) { return !SEGS ? kt * BK : SEG_POW2 ? (kt & (nk_seg - 1)) * BK : (kt % nk_seg) * BK; };
  {
    // A k-tile is two k-steps of 32; a k-step runs in two phases, one per half of the wave's A
    // fragments (MI / 2 x NI MFMAs each), so that only half of them are live at a time.  Phase p uses
    // A buffer p % 2 and B buffer (p / 2) % 2 and fetches the fragments of phase p + 1 meanwhile.
    // One barrier per k-tile, placed between phases 2 and 3.  By then every wave holds its phase-3
    // fragments of the current stage in registers and has written tile kt+1 into the other stage, so
    // after the barrier phase 3's MFMAs run while the first fragments of the NEXT stage are fetched:
    // no LDS latency is exposed behind the barrier.  Within a phase the scheduler is told to
    // alternate one MFMA with one LDS/global access.
    constexpr int MH = MI / 2;
    static_assert(TL::TM % 32 == 0 && TL::TN % 32 == 0, "a wave's sub-tile starts at a multiple of 32");
    KFragLane kl;
    TFragLane<BM> tla;
    TFragLane<BN> tlb;
    kl.init(lane);
    tla.init(lane);
    tlb.init(lane);
    constexpr int NRA = AK ? MH : 2 * MH, NRB = BKC ? NI : 2 * NI;  // LDS reads of an A half / of B
    constexpr int NMMA = MH * NI;
    bf16x8 af[2][MH], bfr[2][NI];
    auto ldA = [&](int buf, const bf16_t* as, int kk, int half) {
#pragma unroll
      for (int i = 0; i < MH; ++i) af[buf][i] = load_frag<AK, BM>(as + wm * TL::TM * (AK ? BK : 1), (half * MH + i) * 16, kk, kl, tla);
    };
    auto ldB = [&](int buf, const bf16_t* bs, int kk) {
#pragma unroll
      for (int j = 0; j < NI; ++j) bfr[buf][j] = load_frag<BKC, BN>(bs + wn * TL::TN * (BKC ? BK : 1), j * 16, kk, kl, tlb);
    };
    auto mma = [&](int abuf, int bbuf, auto half) {
      constexpr int H = decltype(half)::value;
#pragma unroll
      for (int i = 0; i < MH; ++i)
#pragma unroll
        for (int jj = 0; jj < NI; ++jj) {
          // serpentine: one operand changes from one MFMA to the next, never both (on a register-only
          // loop under the power limit 2 % faster than row-major and 5 % than both changing; inside
          // this kernel the difference is within the noise)
          const int j = (i & 1) ? NI - 1 - jj : jj;
          acc[H * MH + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[abuf][i], bfr[bbuf][j], acc[H * MH + i][j], 0, 0, 0);
        }
    };
    // mask: 0x008 MFMA, 0x100 LDS read, 0x200 LDS write, 0x020 global read
    auto interleave2 = [&](auto nread, auto mask1, auto n1, auto mask2, auto n2) {
      constexpr int NREAD = decltype(nread)::value;
#pragma unroll
      for (int i = 0; i < NMMA; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (i * ((NREAD + NMMA - 1) / NMMA) < NREAD) __builtin_amdgcn_sched_group_barrier(0x100, (NREAD + NMMA - 1) / NMMA, 0);
        if (decltype(n1)::value > 0 && i < decltype(n1)::value)
          __builtin_amdgcn_sched_group_barrier(decltype(mask1)::value, 1, 0);
        if (decltype(n2)::value > 0 && i < decltype(n2)::value)
          __builtin_amdgcn_sched_group_barrier(decltype(mask2)::value, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);  // nothing moves across the end of a phase
    };
    typedef std::integral_constant<int, 0x200> MW;
    typedef std::integral_constant<int, 0x020> MG;
    constexpr bool SPLIT = AK;  // staging of A in phase 2 instead of phase 0
    typedef std::integral_constant<int, (SPLIT ? 0 : Stager<AK, BM, NT>::CHUNKS) + Stager<BKC, BN, NT>::CHUNKS> NC0;
    typedef std::integral_constant<int, Stager<AK, BM, NT>::CHUNKS> NC2;
    typedef std::integral_constant<int, 0> N0;
    typedef std::integral_constant<int, NRA> RA;
    typedef std::integral_constant<int, NRA + NRB> RAB;
    typedef std::integral_constant<int, 0> H0;
    typedef std::integral_constant<int, 1> H1;

    sa.load(A, lda, m0, 0);
    sb.load(B, ldb, n0, 0);
    sa.store(smem);
    sb.store(smem + A_ST);
    if (nk > 1) {
      sa.load(seg_a_of(1), lda, m0, k0_of(1));
      sb.load(seg_b_of(1), ldb, n0, k0_of(1));
    }
    __syncthreads();
    ldA(0, smem, 0, 0);
    ldB(0, smem + A_ST, 0);
    auto iter = [&](int kt, auto do_store, auto do_load) {
      const int cur = kt & 1;
      const bf16_t* as = smem + cur * STAGE;
      const bf16_t* bs = as + A_ST;
      const bf16_t* an = smem + (cur ^ 1) * STAGE;
      const bf16_t* bn2 = an + A_ST;
      // phase 0: tile kt+1 (in registers since the previous iteration) goes to the other stage.  With
      // a K-contiguous A (forward, dgrad) only its B part: the A part follows in phase 2, the phase with
      // the fewest fragment reads, so that the phases issue about the same number of memory
      // instructions beside their MFMAs (+2-6 % on the forward products; the weight-gradient layout,
      // all transpose loads, is 2 % faster with everything in phase 0).
      ldA(1, as, 0, 1);
      if constexpr (decltype(do_store)::value) {
        if constexpr (!SPLIT) sa.store(smem + (cur ^ 1) * STAGE);
        sb.store(smem + (cur ^ 1) * STAGE + A_ST);
      }
      // the registers are free again as soon as their LDS store has issued: the loads of tile kt+2
      // follow at once, a full k-tile ahead of their use
      if constexpr (decltype(do_load)::value) {
        if constexpr (!SPLIT) sa.load(seg_a_of(kt + 2), lda, m0, k0_of(kt + 2));
        sb.load(seg_b_of(kt + 2), ldb, n0, k0_of(kt + 2));
      }
      mma(0, 0, H0{});
      if constexpr (decltype(do_load)::value) interleave2(RA{}, MW{}, NC0{}, MG{}, NC0{});
      else if constexpr (decltype(do_store)::value) interleave2(RA{}, MW{}, NC0{}, MW{}, N0{});
      else interleave2(RA{}, MW{}, N0{}, MW{}, N0{});
      // phase 1
      ldA(0, as, 1, 0);
      ldB(1, bs, 1);
      mma(1, 0, H1{});
      interleave2(RAB{}, MW{}, N0{}, MW{}, N0{});
      // phase 2
      ldA(1, as, 1, 1);
      if constexpr (SPLIT && decltype(do_store)::value) sa.store(smem + (cur ^ 1) * STAGE);
      if constexpr (SPLIT && decltype(do_load)::value) sa.load(seg_a_of(kt + 2), lda, m0, k0_of(kt + 2));
      mma(0, 1, H0{});
      if constexpr (SPLIT && decltype(do_load)::value) interleave2(RA{}, MW{}, NC2{}, MG{}, NC2{});
      else if constexpr (SPLIT && decltype(do_store)::value) interleave2(RA{}, MW{}, NC2{}, MW{}, N0{});
      else interleave2(RA{}, MW{}, N0{}, MW{}, N0{});
      __syncthreads();
      // phase 3, overlapped with the fetch of the next stage's first fragments
      ldA(0, an, 0, 0);
      ldB(0, bn2, 0);
      mma(1, 1, H1{});
      interleave2(RAB{}, MW{}, N0{}, MW{}, N0{});
    };
    int kt = 0;
    for (; kt + 2 < nk; ++kt) iter(kt, std::true_type{}, std::true_type{});
    if (kt + 1 < nk) { iter(kt, std::true_type{}, std::false_type{}); ++kt; }
    prefetch_r(std::true_type{});
    iter(kt, std::false_type{}, std::false_type{});
    prefetch_r(std::false_type{});
    __syncthreads();
  }

  if constexpr (EPI == E_ACCUM) {
    // fp32 main-grad: 16 lanes cover 64 contiguous bytes of a row, stored directly
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const size_t row = m0 + wm * TL::TM + i * 16 + (lane >> 4) * 4 + r;
          const size_t col = n0 + wn * TL::TN + j * 16 + (lane & 15);
          C[row * (size_t)N + col] = acc[i][j][r];
        }
  } else {
    // bf16 outputs: the fp32 accumulators pass through LDS, 64 tile rows at a time, so that every
    // thread finishes 8 adjacent columns (bias, residual, GeLU in fp32, one rounding) and the
    // global accesses of C, C2 and R are 16 bytes per lane over whole 512-byte row segments.
    constexpr int LDC = BN + 4;
    float* cs = reinterpret_cast<float*>(smem_raw);
    static_assert((size_t)PR * LDC * 4 <= 2 * (size_t)STAGE * sizeof(bf16_t), "epilogue staging does not fit");
    // E_GELU_BWD with colpart: the column sums of this tile's (rounded) outputs, i.e. the tile's share of the bias
    // gradient of the linear layer whose pre-activation gradient is being written; a thread keeps the sums of
    // its 8 columns over its rows, the threads of a column group meet in LDS after the last pass
    float csum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int p = 0; p < BM / PR; ++p) {
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int r0 = wm * TL::TM + i * 16;
        if (r0 / PR != p) continue;
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            cs[(r0 % PR + (lane >> 4) * 4 + r) * LDC + wn * TL::TN + j * 16 + (lane & 15)] = acc[i][j][r];
      }
      __syncthreads();
#pragma unroll
      for (int q = 0; q < NQ; ++q) {
        const int c = tid + q * NT, lr = c / (BN / 8), lc = (c % (BN / 8)) * 8;
        const size_t row = m0 + p * PR + lr, col = n0 + lc, idx = row * (size_t)N + col;
        float v[8];
        *reinterpret_cast<f32x4*>(v) = *reinterpret_cast<const f32x4*>(cs + lr * LDC + lc);
        *reinterpret_cast<f32x4*>(v + 4) = *reinterpret_cast<const f32x4*>(cs + lr * LDC + lc + 4);
        if constexpr (EPI == E_BIAS || EPI == E_BIAS_RES || EPI == E_BIAS_GELU) {
          const f32x4 b0 = *reinterpret_cast<const f32x4*>(bias + col), b1 = *reinterpret_cast<const f32x4*>(bias + col + 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) { v[e] += b0[e]; v[4 + e] += b1[e]; }
        }
        bf16x8 o;
        if constexpr (EPI == E_BIAS_RES) {
          const bf16x8 rr = rpre[p][q];
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (__bf16)(v[e] + (float)rr[e]);
        } else if constexpr (EPI == E_GELU_BWD) {
          const bf16x8 rr = rpre[p][q];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            o[e] = (__bf16)(v[e] * gelu_grad_f((float)rr[e]));
            csum[e] += (float)o[e];
          }
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (__bf16)v[e];
        }
        *reinterpret_cast<bf16x8*>(C + idx) = o;
        if constexpr (EPI == E_BIAS_GELU) {
          bf16x8 g2;
#pragma unroll
          for (int e = 0; e < 8; ++e) g2[e] = (__bf16)gelu_f((float)o[e]);
          *reinterpret_cast<bf16x8*>(C2 + idx) = g2;
        }
      }
      __syncthreads();
    }
    if constexpr (EPI == E_GELU_BWD) {
      if (colpart) {
        // thread tid owns column group tid % (BN / 8) in every pass (NT is a multiple of BN / 8) and the rows
        // tid / (BN / 8) + k * RG: RG partial sums per column, added in ascending order
        constexpr int CGN = BN / 8, RG = NT / CGN;
        static_assert(NT % CGN == 0 && (size_t)RG * BN * 4 <= 2 * (size_t)STAGE * sizeof(bf16_t), "column-sum staging does not fit");
        const int g = tid % CGN, rg = tid / CGN;
#pragma unroll
        for (int e = 0; e < 8; ++e) cs[rg * BN + g * 8 + e] = csum[e];
        __syncthreads();
        for (int c = tid; c < BN; c += NT) {
          float t = 0.f;
#pragma unroll 8
          for (int r = 0; r < RG; ++r) t += cs[r * BN + c];
          colpart[(size_t)bm * N + n0 + c] = t;
        }
      }
    }
  }
}

typedef Tile<256, 256, 2, 4> TileBig;    // 8 waves, 128 x 64 per wave (8 x 4 MFMA tiles)
typedef Tile<256, 128, 4, 2> TileMid;    // 8 waves, 64 x 64 per wave
typedef Tile<128, 128, 2, 2> TileSmall;  // 4 waves, 64 x 64 per wave
// 8 waves, 64 x 96 per wave, for outputs of 6144 columns (24 times 256, but 32 times 192): 2048 rows are 256 such
// tiles, one round, where 256 x 256 gives 192.  For the forward and dgrad layouts with the one-output epilogues
// (none, bias, bias + residual); the epilogue that also takes column sums needs the threads to divide into the
// tile's 24 column groups and keeps the other shapes.
typedef Tile<256, 192, 4, 2> TileWide;

template <typename TL, bool AK, bool BKC>
constexpr size_t lds_bytes() { return 2 * (size_t)(stage_elems<AK, TL::BM>() + stage_elems<BKC, TL::BN>()) * sizeof(bf16_t); }

template <typename TL, bool AK, bool BKC, int EPI, typename TO, bool SEG_POW2 = false>
bf_status launch(const GemmArgs& a, hipStream_t st) {
  if constexpr (EPI == E_ACCUM && !SEG_POW2) {
    const int nk_seg = a.K / ((AK && a.k_slices > 1) ? a.k_slices : 1) / BK;
    if ((nk_seg & (nk_seg - 1)) == 0) return launch<TL, AK, BKC, EPI, TO, true>(a, st);
  }
  auto kern = gemm_mfma_kernel<TL, AK, BKC, EPI, TO, SEG_POW2>;
  constexpr size_t lds = lds_bytes<TL, AK, BKC>();
  // The LDS reservation is a per-device attribute of the kernel: one bit per device and instantiation,
  // set after the call has succeeded (two threads racing here both make the call, which is harmless).
  static std::atomic<uint64_t> attr_set{0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) { set_error("gemm_mfma: no current device"); return BF_EDEVICE; }
  const uint64_t bit = 1ull << (dev & 63);
  if (dev >= 64 || !(attr_set.load(std::memory_order_acquire) & bit)) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) { set_error("gemm_mfma: cannot reserve %zu bytes of LDS: %s", lds, hipGetErrorString(e)); return BF_EDEVICE; }
    if (dev < 64) attr_set.fetch_or(bit, std::memory_order_release);
  }
  const int tiles_m = a.M / TL::BM, tiles_n = a.N / TL::BN;
  const int remap = (tiles_m * tiles_n) % 8 == 0 ? 1 : 0;
  // split-K (fp32 planes of partial results, forward / dgrad layouts only): a.K is the whole contraction, the kernel
  // gets the slice length and the row length of the K-contiguous operands separately
  const int slices = (EPI == E_ACCUM && AK && a.k_slices > 1) ? a.k_slices : 1;
  const dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)slices);
  kern<<<grid, TL::NT, lds, st>>>(a.M, a.N, a.K / slices, (const bf16_t*)a.A, (const bf16_t*)a.B, (TO*)a.C, a.bias,
                                  (const TO*)a.R, (TO*)a.C2, a.accumulate, tiles_m, remap, a.n_seg > 1 ? a.n_seg : 1,
                                  a.seg_stride_a, a.seg_stride_b, EPI == E_GELU_BWD ? a.colsum_part : nullptr, a.K);
  if (EPI == E_GELU_BWD && a.colsum_rows) *a.colsum_rows = tiles_m;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("gemm_mfma launch failed: %s", hipGetErrorString(e)); return BF_EDEVICE; }
  return BF_OK;
}

template <typename TL, bool AK, bool BKC>
bf_status by_epilogue(int epi, const GemmArgs& a, hipStream_t st) {
  switch (epi) {
    case E_NONE: return launch<TL, AK, BKC, E_NONE, bf16_t>(a, st);
    case E_BIAS: return launch<TL, AK, BKC, E_BIAS, bf16_t>(a, st);
    case E_BIAS_RES: return launch<TL, AK, BKC, E_BIAS_RES, bf16_t>(a, st);
    case E_BIAS_GELU: return launch<TL, AK, BKC, E_BIAS_GELU, bf16_t>(a, st);
    case E_GELU_BWD: return launch<TL, AK, BKC, E_GELU_BWD, bf16_t>(a, st);
    default: break;
  }
  set_error("gemm_mfma: epilogue %d not available for this layout", epi);
  return BF_EINVAL;
}

template <typename TL>
bf_status by_layout(int layout, int epi, const GemmArgs& a, hipStream_t st) {
  if (epi == E_ACCUM && layout != L_TN) {  // fp32 planes of a split contraction
    if (layout == L_NN) return launch<TL, true, false, E_ACCUM, float>(a, st);
    return launch<TL, true, true, E_ACCUM, float>(a, st);
  }
  if (layout == L_NN) return by_epilogue<TL, true, false>(epi, a, st);
  if (layout == L_NT) return by_epilogue<TL, true, true>(epi, a, st);
  if (epi != E_ACCUM) { set_error("gemm_mfma: the weight-gradient layout stores fp32 with E_ACCUM only"); return BF_EINVAL; }
  return launch<TL, false, false, E_ACCUM, float>(a, st);
}

inline bool small_fits(int M, int N) { return M % 128 == 0 && N % 128 == 0; }
inline bool wide_fits(int layout, int epi, int M, int N) {
  if (M % 256 || N % 192) return false;
  if (layout == L_NT) return epi == E_NONE;
  return layout == L_NN && (epi == E_NONE || epi == E_BIAS || epi == E_BIAS_RES);
}
constexpr int SPLITK_TILE = 1;  // split contractions run on the 256 x 128 tile

// Tile choice: the grid runs in rounds over the chip's workgroup slots, so the estimated time of a
// tile shape is rounds x tile area / (throughput of a slot relative to a compute unit running the
// 256 x 256 tile).  Larger tiles reuse more per LDS byte; smaller ones fill the last round.  A
// partly filled last round counts as (1 + fill) / 2 of a round: the chip runs at its power limit,
// and the compute units that do work clock higher when the others idle (measured: 384 large tiles
// beat 768 of 256 x 128, 128 large tiles lose to 256 of them).
// 0: 256 x 256 (one per compute unit), 1: 256 x 128 (one), 2: 128 x 128 (two), 3: 256 x 192 (one; only where the
// caller says the product can take it).
inline int choose_tile(int M, int N, bool wide = false) {
  const int bm[4] = {256, 256, 128, 256}, bn[4] = {256, 128, 128, 192};
  const long slots[4] = {256, 256, 512, 256};
  const double rate[4] = {1.0, TILE_RATE_MID, TILE_RATE_SMALL / 2, TILE_RATE_WIDE};
  int best = -1;
  double best_t = 0;
  for (int i = 0; i < (wide ? 4 : 3); ++i) {
    if (M % bm[i] || N % bn[i]) continue;
    const long tiles = (long)(M / bm[i]) * (N / bn[i]), full = tiles / slots[i], rest = tiles % slots[i];
    const double rounds = (double)full + (rest ? 0.5 + 0.5 * (double)rest / slots[i] : 0.0);
    const double t = rounds * bm[i] * bn[i] / rate[i];
    if (best < 0 || t < best_t) { best = i; best_t = t; }
  }
  return best;
}

}  // namespace

bool gemm_mfma_supported(int layout, int epi, int M, int N, int K) {
  if (layout < L_NN || layout > L_TN) return false;
  if ((layout == L_TN) != (epi == E_ACCUM)) return false;
  if (epi < E_NONE || epi > E_ACCUM) return false;
  if (M < 1 || N < 1 || K < BK || K % BK) return false;
  return small_fits(M, N);
}

void gemm_mfma_tile(int layout, int epi, int M, int N, int* bm, int* bn) {
  const int rows[4] = {256, 256, 128, 256}, cols[4] = {256, 128, 128, 192};
  const int t = choose_tile(M, N, wide_fits(layout, epi, M, N));
  *bm = t < 0 ? 0 : rows[t];
  *bn = t < 0 ? 0 : cols[t];
}

bf_status gemm_mfma(int layout, int epi, const GemmArgs& a, hipStream_t st) {
  const bool planes = epi == E_ACCUM && layout != L_TN;  // split contraction of a forward / dgrad product
  if (planes) {
    if (a.k_slices < 2 || a.K % (a.k_slices * BK) || !gemm_mfma_supported(layout, E_NONE, a.M, a.N, a.K / a.k_slices) || a.accumulate ||
        a.n_seg > 1) {
      set_error("gemm_mfma: bad split of the contraction (%d slices of K = %d)", a.k_slices, a.K);
      return BF_EINVAL;
    }
  } else if (!gemm_mfma_supported(layout, epi, a.M, a.N, a.K)) { set_error("gemm_mfma: shape not supported"); return BF_EINVAL; }
  if (a.n_seg > 1 && (layout != L_TN || ((a.seg_stride_a | a.seg_stride_b) & 7))) {
    set_error("gemm_mfma: segments go with the weight-gradient layout and 16-byte aligned strides");
    return BF_EINVAL;
  }
  const uintptr_t al = (uintptr_t)a.A | (uintptr_t)a.B | (uintptr_t)a.C | (uintptr_t)a.R | (uintptr_t)a.C2 | (uintptr_t)a.bias;
  if (al & 15) { set_error("gemm_mfma: operands must be 16-byte aligned"); return BF_EINVAL; }
  switch (planes ? SPLITK_TILE : choose_tile(a.M, a.N, !a.shared_chip && wide_fits(layout, epi, a.M, a.N))) {
    case 0: return by_layout<TileBig>(layout, epi, a, st);
    case 1: return by_layout<TileMid>(layout, epi, a, st);
    case 3:
      if (layout == L_NT) return launch<TileWide, true, true, E_NONE, bf16_t>(a, st);
      if (epi == E_BIAS) return launch<TileWide, true, false, E_BIAS, bf16_t>(a, st);
      if (epi == E_BIAS_RES) return launch<TileWide, true, false, E_BIAS_RES, bf16_t>(a, st);
      return launch<TileWide, true, false, E_NONE, bf16_t>(a, st);
    default: return by_layout<TileSmall>(layout, epi, a, st);
  }
}

// Split-K.  A product whose best tile shape still leaves half of the workgroup slots of its only round empty (the
// 2048-column products of a 2048-wide model on 2048-row micro-batches: 128 tiles of 256 x 128) runs its contraction
// in two slices on twice as many workgroups; each slice leaves an fp32 plane and a second kernel adds the planes in
// ascending order and applies the epilogue, so the result does not depend on which slice finishes first.  Measured on
// the step of a 2048-wide, 6-layer model (8 micro-batches of 2048 rows): 48.8 -> 44.6 ms with K >= 4096 split, 44.3 with
// K >= 2048; four slices on 256 x 256 tiles instead: 45.6.
int gemm_splitk_slices(int layout, int epi, int M, int N, int K) {
  if (layout != L_NN && layout != L_NT) return 1;
  if (epi != E_NONE && epi != E_BIAS && epi != E_BIAS_RES) return 1;
  if (K < 2048 || K % (2 * BK) || !gemm_mfma_supported(layout, epi, M, N, K)) return 1;
  if (M % 256 || N % 128) return 1;
  if (choose_tile(M, N) != SPLITK_TILE) return 1;
  const long tiles = (long)(M / 256) * (N / 128);
  return tiles <= 128 ? 2 : 1;
}

}  // namespace bf
