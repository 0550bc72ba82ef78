// Fused attention on the gfx950 matrix cores: softmax(Q K^T / sqrt(S_head) [+ causal mask]) V
// forward, and its backward as two deterministic passes (dQ pass over key blocks, dK/dV pass
// over query blocks) that recompute the probabilities from the saved log-sum-exp.  No
// S_seq x S_seq tensor ever reaches HBM and nothing is accumulated with atomics, so the
// result does not depend on scheduling.
//
// Every score tile is computed TRANSPOSED where that keeps "one lane = one softmax row":
//   forward / dQ pass:  S^T = K Q^T   (MFMA rows = keys,    columns = the wave's 32 queries)
//   dK/dV pass:         S   = Q K^T   (MFMA rows = queries, columns = the wave's 32 keys)
// In the accumulator layout of v_mfma_f32_32x32x16_bf16 (lane l, register r holds
// row (r/4)*8 + (l/32)*4 + r%4, column l%32) a lane then owns one column and 16 rows, so a
// row statistic of the softmax is a per-lane scalar (forward) and the 8 registers
// 8kk..8kk+7 of a lane, rounded to bf16, are directly the B operand of the next product
// for the contraction rows 16kk + 8(e/4) + 4(l/32) + e%4.  The matching A operand is read
// from LDS with the transpose load (ds_read_b64_tr_b16) using that same row order.
//
// LDS tiles are [row][S_head] with the 16-byte chunk index XOR-swizzled by row bits; the
// layout serves both the K-contiguous 16-byte fragment reads and the transpose loads without
// bank conflicts.
#include <type_traits>

#include "common.h"

namespace bf {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int NTHR = 256;   // 4 waves; wave w owns rows 32w..32w+31 of the workgroup's 128-row block
constexpr int WG_ROWS = 128;
constexpr int BLK = 64;     // rows of the streamed tiles (keys in forward/dQ, queries in dK/dV)
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

// XOR key of a tile row.  The LDS has 64 banks of 4 bytes; a 16-byte-per-lane read is served 16
// lanes (16 rows, one logical chunk) at a time and a transpose load 32 lanes (4 rows x 4
// adjacent chunks) at a time.  Both sets land in 16 distinct 16-byte slots of the 256-byte bank
// line when the key sends row bits 0-1 to chunk bits 2-3 and row bits 2-3 to chunk bits 0-1
// (S_head 128: 16 chunks per 256-byte row), or row bit 1 to chunk bit 2 and row bits 2-3 to chunk
// bits 0-1 with the row parity choosing the half line (S_head 64: 8 chunks per 128-byte row).
template <int D>
__device__ __forceinline__ int row_key(int row) {
  return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}

template <int D>
__device__ __forceinline__ int swz(int row, int col) {
  return row * D + ((((col >> 3) ^ row_key<D>(row)) << 3) | (col & 7));
}

// thread's 16-byte chunks of a [ROWS][D] tile
template <int ROWS, int D, int NT = 256>
struct TileRegs {
  static constexpr int CH = ROWS * D / 8 / NT;
  u32x4 v[CH];
  __device__ __forceinline__ void load(const bf16_t* __restrict__ g, size_t ld, int tid) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = tid + i * NT, row = c / (D / 8), ch = c % (D / 8);
      v[i] = *reinterpret_cast<const u32x4*>(g + (size_t)row * ld + ch * 8);
    }
  }
  __device__ __forceinline__ void store(bf16_t* lds, int tid) const {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = tid + i * NT, row = c / (D / 8), ch = c % (D / 8);
      *reinterpret_cast<u32x4*>(lds + row * D + ((ch ^ row_key<D>(row)) << 3)) = v[i];
    }
  }
};

// A operand, contraction along the tile's columns: lane holds tile[row0 + l%32][16kk + 8(l/32) .. +7]
template <int D>
__device__ __forceinline__ bf16x8 frag_k(const bf16_t* tile, int row0, int kk, int lane) {
  return *reinterpret_cast<const bf16x8*>(tile + swz<D>(row0 + (lane & 31), kk * 16 + 8 * (lane >> 5)));
}

// A operand, contraction along the tile's rows in the accumulator order: lane holds
// tile[rowbase + 8(e/4) + 4(l/32) + e%4][col0 + l%32] for e = 0..7
template <int D>
__device__ __forceinline__ bf16x8 frag_t(const bf16_t* tile, int rowbase, int col0, int lane) {
  const int t = lane & 15, blk = lane >> 4;
  const int row = rowbase + 4 * (blk >> 1) + (t >> 2);
  const int col = col0 + 16 * (blk & 1) + 4 * (t & 3);
  typedef s16x4 __attribute__((address_space(3))) * lds_v4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(tile + swz<D>(row, col)));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(tile + swz<D>(row + 8, col)));
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// registers 8kk..8kk+7 of an accumulator tile as a bf16 B operand
__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int kk) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (__bf16)a[8 * kk + e];
  return o;
}

// B operand straight from global memory: lane holds row[16kk + 8(l/32) .. +7] of its own token row
template <int D>
__device__ __forceinline__ void load_rowfrags(const bf16_t* __restrict__ row, int lane, bf16x8 (&f)[D / 16]) {
#pragma unroll
  for (int kk = 0; kk < D / 16; ++kk) f[kk] = *reinterpret_cast<const bf16x8*>(row + kk * 16 + 8 * (lane >> 5));
}

// Scheduling hint for a run of NMMA MFMAs that each consume RPM LDS reads: the reads run AHEAD
// MFMAs in front of their use (an LDS read takes a few MFMA times to return), then nothing moves
// across the end of the run.
template <int NMMA, int RPM, int AHEAD>
__device__ __forceinline__ void mfma_lds_pipeline() {
  __builtin_amdgcn_sched_group_barrier(0x100, AHEAD * RPM, 0);
#pragma unroll
  for (int i = 0; i < NMMA - AHEAD; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);
  }
  __builtin_amdgcn_sched_group_barrier(0x008, AHEAD, 0);
  __builtin_amdgcn_sched_barrier(0);
}

__device__ __forceinline__ int acc_row(int r, int lane) { return (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3); }

__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}

// store a transposed accumulator set acc[dt] (rows = head dims, column = this lane's token) as a token row
template <int D>
__device__ __forceinline__ void store_rows(const f32x16 (&acc)[D / 32], bf16_t* __restrict__ row, int lane, float mul) {
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (__bf16)(acc[dt][q4 * 4 + e] * mul);
      *reinterpret_cast<bf16x4*>(row + dt * 32 + q4 * 8 + (lane >> 5) * 4) = o;
    }
}

// ---- column sums of a transposed accumulator set over a workgroup's tokens (the bias gradient of the QKV
// projection is the column sum of dqkv: taking it here saves a second pass over that tensor).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  const int i = __builtin_bit_cast(int, v);  // every lane has a source under these controls: `old` is never taken
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(i, i, CTRL, 0xf, 0xf, true));
}
// every lane gets the sum over its row of 16 lanes: neighbours in a quad, the other pair of the quad, the
// mirrored half of 8, the mirrored half of 16
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_f32<0xB1>(v);   // quad_perm [1, 0, 3, 2]
  v += dpp_f32<0x4E>(v);   // quad_perm [2, 3, 0, 1]
  v += dpp_f32<0x141>(v);  // row_half_mirror
  v += dpp_f32<0x140>(v);  // row_mirror
  return v;
}
// acc[dt][r] of lane l is head dimension 32 dt + acc_row(r, l) of token l % 32.  The wave leaves the sums over
// each of its four rows of 16 lanes in red[row][16 dt + r] (rows 0-1: lanes 0-31, rows 2-3: lanes 32-63).
template <int D>
__device__ __forceinline__ void wave_colsum(const f32x16 (&acc)[D / 32], float mul, float* red, int lane) {
  f32x16 v[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) v[dt][r] = row16_sum(acc[dt][r] * mul);
  if ((lane & 15) == 0) {  // one lane per row stores the row's D / 2 sums, 16 bytes at a time
    typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
    f32x4* dst = reinterpret_cast<f32x4*>(red + (lane >> 4) * (D / 2));
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = v[dt][q4 * 4 + e];
        dst[dt * 4 + q4] = o;
      }
  }
}
// head dimension d of the workgroup's column sums: waves w0 .. w0 + nw - 1 of red ([wave][4][D / 2]) in order
template <int D>
__device__ __forceinline__ float colsum_of(const float* red, int w0, int nw, int d) {
  const int dt = d >> 5, rem = d & 31, r = ((rem >> 3) << 2) | (rem & 3), hh = (rem >> 2) & 1;
  float t = 0.f;
  for (int w = w0; w < w0 + nw; ++w) {
    const float* rw = red + (size_t)w * 4 * (D / 2) + dt * 16 + r;
    t += rw[(2 * hh) * (D / 2)] + rw[(2 * hh + 1) * (D / 2)];
  }
  return t;
}

// Per-lane LDS offsets of the fragment reads.  The XOR swizzle makes an address a non-linear
// function of (row, chunk), but the key depends on the lane's row modulo 16 only, so a lane has one
// offset per distinct chunk pattern; tile row blocks of 16 / 32 rows and the LDS stage then enter as
// compile-time constants that the DS instructions take as immediates instead of a shift / xor / add
// chain per read.
template <int D>
struct FragAddr {
  int k[D / 16];      // frag_k, rows 0-31: element offset of chunk 2kk + lane/32 of row lane%32
  int t[2][D / 32];   // frag_t, row block 0: offsets of the two transpose loads (rows r, r+8) per 32-column block
  __device__ __forceinline__ void init(int lane) {
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) k[kk] = swz<D>(lane & 31, kk * 16 + 8 * (lane >> 5));
    const int tt = lane & 15, blk = lane >> 4;
    const int row = 4 * (blk >> 1) + (tt >> 2), col = 16 * (blk & 1) + 4 * (tt & 3);
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
      t[0][dt] = swz<D>(row, 32 * dt + col);
      t[1][dt] = swz<D>(row + 8, 32 * dt + col);
    }
  }
  // A operand, contraction along the tile's columns: lane holds tile[row0 + l%32][16kk + 8(l/32) .. +7]; row0 % 16 == 0
  __device__ __forceinline__ bf16x8 frag_k(const bf16_t* tile, int row0, int kk) const {
    return *reinterpret_cast<const bf16x8*>(tile + row0 * D + k[kk]);
  }
  // A operand, contraction along the tile's rows in the accumulator order: lane holds
  // tile[rowbase + 8(e/4) + 4(l/32) + e%4][32 dt + l%32] for e = 0..7; rowbase % 16 == 0
  __device__ __forceinline__ bf16x8 frag_t(const bf16_t* tile, int rowbase, int dt) const {
    typedef s16x4 __attribute__((address_space(3))) * lds_v4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(tile + rowbase * D + t[0][dt]));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(tile + rowbase * D + t[1][dt]));
    return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  }
};

// The same interface computing every address on the fly: for kernels that have no 16 registers to spare.
template <int D>
struct FragAddrLive {
  int lane_;
  __device__ __forceinline__ void init(int lane) { lane_ = lane; }
  __device__ __forceinline__ bf16x8 frag_k(const bf16_t* tile, int row0, int kk) const { return bf::frag_k<D>(tile, row0, kk, lane_); }
  __device__ __forceinline__ bf16x8 frag_t(const bf16_t* tile, int rowbase, int dt) const { return bf::frag_t<D>(tile, rowbase, 32 * dt, lane_); }
};

// Register set that carries tile j+1, from the parity of j: a compile-time constant when the loop
// is unrolled by two (the parity is an integral_constant), always set 0 with one tile in flight.
template <int DEPTH, typename P>
struct NextSetOf { static constexpr int value = 0; };
template <int DEPTH, int V>
struct NextSetOf<DEPTH, std::integral_constant<int, V>> { static constexpr int value = (V + 1) % DEPTH; };

// ------------------------------------------------------------------------------ forward
// ROWS queries per workgroup (one wave per 32): 128 with 4 waves and two workgroups per compute
// unit, or 256 with 8 waves and one.  The K/V tiles come through registers DEPTH tiles ahead of
// their use and are double-buffered in LDS: tile j+1 is written to the idle stage while tile j is
// consumed, so an iteration has a single barrier.  The 256-query form reads each tile from HBM / L2
// once for twice as many queries and keeps two tiles in flight; it needs enough (head, block) pairs
// to fill the chip.
// Measured at S_seq 1024-2048, 64 heads of 128: timed without softmax, P V and K/V refetch, the bare
// S = K Q^T loop (one 1 KB LDS fragment read per MFMA, Q from registers) reaches 44 % of the MFMA
// rate; without P V 70 % of the full time remains, without the softmax arithmetic 84 %, without the
// K/V refetch 86 %: no single part dominates, the per-tile chain read -> MFMA -> softmax -> MFMA is
// what two wavefronts per SIMD cannot hide.  Fewer LDS bytes per MFMA need 64 queries per wavefront
// (accumulators in AGPRs, one wavefront per SIMD): built and measured level with this form (100 against
// 98 us at 64 heads of 128, S_seq 2048): a lone wavefront issues in order, so each of its LDS, barrier
// and softmax waits stops its MFMAs too, and there is no partner on the SIMD to fill the gap.
template <int D, int ROWS>
__global__ __launch_bounds__(2 * ROWS, ROWS == 128 ? 2 : 1) void attn_fwd_kernel(const bf16_t* __restrict__ qkv,
                                                                                 bf16_t* __restrict__ ctx, float* __restrict__ lse,
                                                                                 int S_seq, int N_heads, int S_mb, int causal,
                                                                                 float scale) {
  constexpr int NT = 2 * ROWS, DEPTH = ROWS == 128 ? 1 : 2;
  __shared__ __attribute__((aligned(16))) bf16_t KVs[2][2][BLK * D];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  // 1-D grid ordered by work: the last (longest) query block of every head first, then the next ...
  const int nhb = N_heads * S_mb;
  const int qblk = S_seq / ROWS - 1 - blockIdx.x / nhb;
  const int head = (blockIdx.x % nhb) % N_heads, b = (blockIdx.x % nhb) / N_heads;
  const int h = N_heads * D;
  const size_t ld = 3 * (size_t)h;
  const bf16_t* base = qkv + (size_t)b * S_seq * ld + head * D;
  const int q0 = qblk * ROWS, qw = q0 + 32 * w, q = qw + (lane & 31);

  FragAddr<D> fa;
  fa.init(lane);
  bf16x8 qf[D / 16];
  load_rowfrags<D>(base + (size_t)q * ld, lane, qf);
  f32x16 o[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) o[dt] = zero16();
  float m = -INFINITY, l = 0.f;
  const float c2 = scale * LOG2E;

  const int nblk = causal ? (q0 + ROWS) / BLK : S_seq / BLK;
  TileRegs<BLK, D, NT> kr[DEPTH], vr[DEPTH];  // set (j % DEPTH) carries tile j
  auto fetch = [&](auto setc, int j) {
    constexpr int SET = decltype(setc)::value;
    kr[SET].load(base + (size_t)j * BLK * ld + h, ld, tid);
    vr[SET].load(base + (size_t)j * BLK * ld + 2 * h, ld, tid);
  };
  typedef std::integral_constant<int, 0> I0;
  typedef std::integral_constant<int, 1> I1;
  fetch(I0{}, 0);
  kr[0].store(KVs[0][0], tid);
  vr[0].store(KVs[0][1], tid);
  if (nblk > 1) fetch(std::integral_constant<int, 1 % DEPTH>{}, 1);
  if (DEPTH > 1 && nblk > 2) fetch(I0{}, 2);
  __syncthreads();
  // one key tile; PAR = j & 1 is a compile-time constant (the loop is unrolled by two) so that the
  // LDS stage and the register set are too
  auto body = [&](int j, auto parc) {
    constexpr int PAR = decltype(parc)::value;
    typedef std::integral_constant<int, (PAR + 1) % DEPTH> NextSet;
    const bf16_t* Ks = KVs[PAR][0];
    const bf16_t* Vs = KVs[PAR][1];
    if (j + 1 < nblk) {
      kr[NextSet::value].store(KVs[PAR ^ 1][0], tid);
      vr[NextSet::value].store(KVs[PAR ^ 1][1], tid);
    }
    if (j + 1 + DEPTH < nblk) fetch(NextSet{}, j + 1 + DEPTH);
    const int kb = j * BLK;
    if (causal && kb > qw + 31) { __syncthreads(); return; }  // the whole tile is above this wave's diagonal
    f32x16 s[2] = {zero16(), zero16()};
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
      for (int t = 0; t < 2; ++t)
        s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.frag_k(Ks, 32 * t, kk), qf[kk], s[t], 0, 0, 0);
    mfma_lds_pipeline<2 * (D / 16), 1, 4>();
    // Online softmax on the raw scores: m is the running max of the unscaled scores, the scale
    // 1/sqrt(S_head) log2(e) enters through one fma per element, the exponentials are the
    // hardware exp2 (arguments <= 0; masked scores are -inf and give exactly 0).
    if (causal && kb + BLK - 1 > qw) {  // only tiles that touch the diagonal pay for the mask
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (kb + 32 * t + acc_row(r, lane) > q) s[t][r] = -INFINITY;
    }
    float mx = m;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[t][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float nmx = -mx * c2;
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[t][r], c2, nmx));
        s[t][r] = p;
        sum += p;
      }
    if (__builtin_amdgcn_ballot_w64(mx > m) != 0) {  // some row's max moved: rescale (rare after the first tiles)
      const float alpha = __builtin_amdgcn_exp2f(fmaf(m, c2, nmx));
      l *= alpha;
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
      m = mx;
    }
    l += sum;
    bf16x8 pb[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2) pb[t][k2] = pack8(s[t], k2);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.frag_t(Vs, 32 * t + 16 * k2, dt), pb[t][k2], o[dt], 0, 0, 0);
    mfma_lds_pipeline<4 * (D / 32), 2, 4>();
    __syncthreads();
  };
  for (int j = 0; j < nblk; j += 2) {
    body(j, I0{});
    if (j + 1 < nblk) body(j + 1, I1{});
  }
  l += __shfl_xor(l, 32, 64);
  store_rows<D>(o, ctx + ((size_t)b * S_seq + q) * h + head * D, lane, 1.0f / l);
  if (lane < 32) lse[((size_t)b * N_heads + head) * S_seq + q] = m * scale + logf(l);
}

// ------------------------------------------------------------------- backward, dQ pass
// Also takes delta[b, head, i] = sum_c dctx[i, c] ctx[i, c] of its queries (each lane already holds
// half of its query's dctx row) and leaves it in `delta` for the dK/dV pass.
// ROWS queries per workgroup and K/V tiles DEPTH tiles ahead, as in the forward kernel.
template <int D, int ROWS>
__global__ __launch_bounds__(2 * ROWS, ROWS == 128 ? 2 : 1) void attn_bwd_dq_kernel(
    const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ ctx, const bf16_t* __restrict__ dctx,
    const float* __restrict__ lse, float* __restrict__ delta, bf16_t* __restrict__ dqkv, int S_seq, int N_heads, int S_mb,
    int causal, float scale, float* __restrict__ colpart) {
  constexpr int NT = 2 * ROWS, DEPTH = ROWS == 128 ? 1 : 2;
  __shared__ __attribute__((aligned(16))) bf16_t KVs[2][2][BLK * D];  // double-buffered, one barrier per tile
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int nhb = N_heads * S_mb;
  const int qblk = S_seq / ROWS - 1 - blockIdx.x / nhb;  // longest query blocks of every head first
  const int head = (blockIdx.x % nhb) % N_heads, b = (blockIdx.x % nhb) / N_heads;
  const int h = N_heads * D;
  const size_t ld = 3 * (size_t)h;
  const bf16_t* base = qkv + (size_t)b * S_seq * ld + head * D;
  const int q0 = qblk * ROWS, qw = q0 + 32 * w, q = qw + (lane & 31);

  // precomputed offsets where the registers allow (the 128-query form at S_head 128 would spill)
  typename std::conditional<(ROWS == 256 || D == 64), FragAddr<D>, FragAddrLive<D>>::type fa;
  fa.init(lane);
  bf16x8 qf[D / 16], dof[D / 16];
  load_rowfrags<D>(base + (size_t)q * ld, lane, qf);
  load_rowfrags<D>(dctx + ((size_t)b * S_seq + q) * h + head * D, lane, dof);
  const size_t st = ((size_t)b * N_heads + head) * S_seq + q;
  float dl = 0.f;
  {
    bf16x8 cf[D / 16];
    load_rowfrags<D>(ctx + ((size_t)b * S_seq + q) * h + head * D, lane, cf);
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
      for (int e = 0; e < 8; ++e) dl = fmaf((float)dof[kk][e], (float)cf[kk][e], dl);
    dl += __shfl_xor(dl, 32, 64);  // lanes l and l + 32 hold the two halves of the row
    if (lane < 32) delta[st] = dl;
  }
  const float lse2 = lse[st] * LOG2E, c2 = scale * LOG2E;
  f32x16 dq[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) dq[dt] = zero16();

  const int nblk = causal ? (q0 + ROWS) / BLK : S_seq / BLK;
  TileRegs<BLK, D, NT> kr[DEPTH], vr[DEPTH];  // set (j % DEPTH) carries tile j
  auto fetch = [&](auto setc, int j) {
    constexpr int SET = decltype(setc)::value;
    kr[SET].load(base + (size_t)j * BLK * ld + h, ld, tid);
    vr[SET].load(base + (size_t)j * BLK * ld + 2 * h, ld, tid);
  };
  typedef std::integral_constant<int, 0> I0;
  typedef std::integral_constant<int, 1> I1;
  fetch(I0{}, 0);
  kr[0].store(KVs[0][0], tid);
  vr[0].store(KVs[0][1], tid);
  if (nblk > 1) fetch(std::integral_constant<int, 1 % DEPTH>{}, 1);
  if (DEPTH > 1 && nblk > 2) fetch(I0{}, 2);
  __syncthreads();
  // one key tile; par = j & 1 selects the LDS stage
  auto body = [&](int j, auto par) {
    typedef std::integral_constant<int, NextSetOf<DEPTH, decltype(par)>::value> NextSet;
    const int p = par;
    const bf16_t* Ks = KVs[p][0];
    const bf16_t* Vs = KVs[p][1];
    if (j + 1 < nblk) {
      kr[NextSet::value].store(KVs[p ^ 1][0], tid);
      vr[NextSet::value].store(KVs[p ^ 1][1], tid);
    }
    if (j + 1 + DEPTH < nblk) fetch(NextSet{}, j + 1 + DEPTH);
    const int kb = j * BLK;
    if (causal && kb > qw + 31) { __syncthreads(); return; }
    const bool diag = causal && kb + BLK - 1 > qw;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16 s = zero16(), dp = zero16();
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kk = 0; kk < D / 16; ++kk) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.frag_k(Ks, 32 * t, kk), qf[kk], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.frag_k(Vs, 32 * t, kk), dof[kk], dp, 0, 0, 0);
      }
      mfma_lds_pipeline<2 * (D / 16), 1, 4>();
      // p = exp(s/sqrt(d) - lse); dS = p (dP - delta) (the factor 1/sqrt(d) is applied once, to dQ)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_exp2f(fmaf(s[r], c2, -lse2)) * (dp[r] - dl);
      if (diag) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (kb + 32 * t + acc_row(r, lane) > q) s[r] = 0.f;
      }
      const bf16x8 dsb[2] = {pack8(s, 0), pack8(s, 1)};
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
        for (int dt = 0; dt < D / 32; ++dt)
          dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.frag_t(Ks, 32 * t + 16 * k2, dt), dsb[k2], dq[dt], 0, 0, 0);
      mfma_lds_pipeline<2 * (D / 32), 2, 4>();
    }
    __syncthreads();
  };
  if constexpr (ROWS == 256 || D == 64) {
    // unrolled by two: the LDS stage (and with it every fragment address) is a compile-time constant
    for (int j = 0; j < nblk; j += 2) {
      body(j, I0{});
      if (j + 1 < nblk) body(j + 1, I1{});
    }
  } else {
    static_assert(DEPTH == 1, "a run-time stage goes with one tile in flight");
    for (int j = 0; j < nblk; ++j) body(j, j & 1);
  }
  store_rows<D>(dq, dqkv + ((size_t)b * S_seq + q) * ld + head * D, lane, scale);
  if (colpart) {
    // row (b, query block) of the partial column sums of dQ, [S_mb * S_seq / ROWS][N_heads * D]; the tile
    // buffers are free: the loop ended on a barrier
    float* red = reinterpret_cast<float*>(&KVs[0][0][0]);
    wave_colsum<D>(dq, scale, red + (size_t)w * 4 * (D / 2), lane);
    __syncthreads();
    if (tid < D) colpart[((size_t)b * (S_seq / ROWS) + qblk) * h + head * D + tid] = colsum_of<D>(red, 0, NT / 64, tid);
  }
}

// ----------------------------------------------------------------- backward, dK/dV pass
// 8 waves per 128-key block, in pairs: waves 0-3 (one per 32 keys) accumulate dV = P^T dO, waves 4-7 the
// matching dK = dS^T Q.  The pair shares the probabilities: the dV wave computes S = Q K^T and
// P = exp(S / sqrt(d) - lse), keeps P (rounded to bf16, as its MFMA operand) and hands it to its
// partner through LDS, lane to lane (both hold the same 32 x 32 accumulator layout); the dK wave
// computes dP = dO V^T meanwhile and forms dS = P (dP - delta).  Each role runs two score-sized
// products per sub-tile and holds one 32 x S_head accumulator set plus its own K or V rows in
// registers, which leaves room for precomputed fragment addresses: two waves share a SIMD and one
// role's exponentials overlap the other's MFMAs.
constexpr int NTHR_DKV = 512;

template <int D>
__global__ __launch_bounds__(NTHR_DKV) void attn_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dctx,
                                                                const float* __restrict__ lse, const float* __restrict__ delta,
                                                                bf16_t* __restrict__ dqkv, int S_seq, int N_heads, int S_mb, int causal,
                                                                float scale, float* __restrict__ colpart) {
  __shared__ __attribute__((aligned(16))) bf16_t QOs[2][2][BLK * D];  // Q and dO tiles, double-buffered
  __shared__ __attribute__((aligned(16))) float stat_s[2][2][BLK];    // lse * log2(e) and delta of the tile's queries
  __shared__ __attribute__((aligned(16))) bf16_t Ps[2][4][2][64 * 8]; // P of a sub-tile: [sub-tile][key group][register half][lane]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int kg = w & 3;
  const bool dk_role = w >= 4;  // wave-uniform
  const int nhb = N_heads * S_mb;
  const int kblk = blockIdx.x / nhb;  // earliest keys see the most queries: those blocks of every head go first
  const int head = (blockIdx.x % nhb) % N_heads, b = (blockIdx.x % nhb) / N_heads;
  const int h = N_heads * D;
  const size_t ld = 3 * (size_t)h;
  const bf16_t* base = qkv + (size_t)b * S_seq * ld + head * D;
  const bf16_t* dob = dctx + (size_t)b * S_seq * h + head * D;
  const float* lrow = lse + ((size_t)b * N_heads + head) * S_seq;
  const float* drow = delta + ((size_t)b * N_heads + head) * S_seq;
  const int k0 = kblk * WG_ROWS, kw = k0 + 32 * kg, key = kw + (lane & 31);

  FragAddr<D> fa;
  fa.init(lane);
  bf16x8 kvf[D / 16];  // this wave's K rows (dV role) or V rows (dK role): the B operand of its score-sized product
  load_rowfrags<D>(base + (size_t)key * ld + (dk_role ? 2 * h : h), lane, kvf);
  const float c2 = scale * LOG2E;
  f32x16 acc[D / 32];  // dV (waves 0-3) or dK (waves 4-7), transposed: rows = head dims, column = key
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) acc[dt] = zero16();

  const int jbeg = causal ? k0 / BLK : 0, nblk = S_seq / BLK;
  TileRegs<BLK, D, NTHR_DKV> qr, dor;
  qr.load(base + (size_t)jbeg * BLK * ld, ld, tid);
  dor.load(dob + (size_t)jbeg * BLK * h, h, tid);
  float lnext = 0.f, dnext = 0.f;
  if (tid < BLK) { lnext = lrow[jbeg * BLK + tid] * LOG2E; dnext = drow[jbeg * BLK + tid]; }
  qr.store(QOs[0][0], tid);
  dor.store(QOs[0][1], tid);
  if (tid < BLK) { stat_s[0][0][tid] = lnext; stat_s[0][1][tid] = dnext; }
  if (jbeg + 1 < nblk) {
    qr.load(base + (size_t)(jbeg + 1) * BLK * ld, ld, tid);
    dor.load(dob + (size_t)(jbeg + 1) * BLK * h, h, tid);
    if (tid < BLK) { lnext = lrow[(jbeg + 1) * BLK + tid] * LOG2E; dnext = drow[(jbeg + 1) * BLK + tid]; }
  }
  __syncthreads();
  // Every wave passes the same barriers per query tile: one per hand-over of P and one at the end
  // (the other LDS stage is complete, this one may be overwritten).
  for (int j = jbeg; j < nblk; ++j) {
    const int cur = (j - jbeg) & 1;
    const bf16_t* Qs = QOs[cur][0];
    const bf16_t* dOs = QOs[cur][1];
    const float* lse_s = stat_s[cur][0];
    const float* delta_s = stat_s[cur][1];
    if (j + 1 < nblk) {
      qr.store(QOs[cur ^ 1][0], tid);
      dor.store(QOs[cur ^ 1][1], tid);
      if (tid < BLK) { stat_s[cur ^ 1][0][tid] = lnext; stat_s[cur ^ 1][1][tid] = dnext; }
    }
    if (j + 2 < nblk) {
      qr.load(base + (size_t)(j + 2) * BLK * ld, ld, tid);
      dor.load(dob + (size_t)(j + 2) * BLK * h, h, tid);
      if (tid < BLK) { lnext = lrow[(j + 2) * BLK + tid] * LOG2E; dnext = drow[(j + 2) * BLK + tid]; }
    }
    const int qb = j * BLK;
    // every query of the tile is before this pair's keys: nothing to add (the partner skips as well)
    const bool skip = causal && qb + BLK - 1 < kw;
    const bool diag = causal && qb < kw + 31;
    // Sub-tiles T0 .. T1-1 (32 queries each) go through the two stages together; every wave passes the
    // hand-over barrier between the stages, whether it has work or not.
    auto stages = [&](auto t0, auto t1) {
      constexpr int T0 = decltype(t0)::value, NTT = decltype(t1)::value - T0;
      bf16x8 pb[NTT][2];
      f32x16 s[NTT];  // S, then P (dV role); dP, then dS (dK role)
#pragma unroll
      for (int u = 0; u < NTT; ++u) s[u] = zero16();
      if (!skip) {
        __builtin_amdgcn_sched_barrier(0);
        if (!dk_role) {
#pragma unroll
          for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
            for (int u = 0; u < NTT; ++u)
              s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.frag_k(Qs, 32 * (T0 + u), kk), kvf[kk], s[u], 0, 0, 0);
          mfma_lds_pipeline<NTT * (D / 16), 1, 4>();
          // P = exp(S / sqrt(d) - lse)
#pragma unroll
          for (int u = 0; u < NTT; ++u) {
            const int t = T0 + u;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[u][r] = __builtin_amdgcn_exp2f(fmaf(s[u][r], c2, -lse_s[32 * t + acc_row(r, lane)]));
            if (diag) {
#pragma unroll
              for (int r = 0; r < 16; ++r)
                if (key > qb + 32 * t + acc_row(r, lane)) s[u][r] = 0.f;
            }
            pb[u][0] = pack8(s[u], 0);
            pb[u][1] = pack8(s[u], 1);
            *reinterpret_cast<bf16x8*>(&Ps[t][kg][0][lane * 8]) = pb[u][0];
            *reinterpret_cast<bf16x8*>(&Ps[t][kg][1][lane * 8]) = pb[u][1];
          }
        } else {
          // dP = dO V^T
#pragma unroll
          for (int kk = 0; kk < D / 16; ++kk)
#pragma unroll
            for (int u = 0; u < NTT; ++u)
              s[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.frag_k(dOs, 32 * (T0 + u), kk), kvf[kk], s[u], 0, 0, 0);
          mfma_lds_pipeline<NTT * (D / 16), 1, 4>();
        }
      }
      __syncthreads();
      if (!skip) {
        if (!dk_role) {
          // dV += dO^T P
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int u = 0; u < NTT; ++u)
#pragma unroll
            for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
              for (int dt = 0; dt < D / 32; ++dt)
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.frag_t(dOs, 32 * (T0 + u) + 16 * k2, dt), pb[u][k2], acc[dt], 0, 0, 0);
          mfma_lds_pipeline<NTT * 2 * (D / 32), 2, 4>();
        } else {
          // dS = P (dP - delta) (the factor 1/sqrt(d) is applied once, to dK; masked entries of P are zero);  dK += Q^T dS
#pragma unroll
          for (int u = 0; u < NTT; ++u) {
            const int t = T0 + u;
            pb[u][0] = *reinterpret_cast<const bf16x8*>(&Ps[t][kg][0][lane * 8]);
            pb[u][1] = *reinterpret_cast<const bf16x8*>(&Ps[t][kg][1][lane * 8]);
#pragma unroll
            for (int r = 0; r < 16; ++r)
              s[u][r] = (float)pb[u][r >> 3][r & 7] * (s[u][r] - delta_s[32 * t + acc_row(r, lane)]);
            pb[u][0] = pack8(s[u], 0);
            pb[u][1] = pack8(s[u], 1);
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int u = 0; u < NTT; ++u)
#pragma unroll
            for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
              for (int dt = 0; dt < D / 32; ++dt)
                acc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa.frag_t(Qs, 32 * (T0 + u) + 16 * k2, dt), pb[u][k2], acc[dt], 0, 0, 0);
          mfma_lds_pipeline<NTT * 2 * (D / 32), 2, 4>();
        }
      }
    };
    typedef std::integral_constant<int, 0> T_0;
    typedef std::integral_constant<int, 1> T_1;
    typedef std::integral_constant<int, 2> T_2;
    if constexpr (D == 128) {
      // both sub-tiles together: two independent accumulators in the score-sized products, one
      // hand-over barrier per tile (measured: 2 % faster than one sub-tile at a time at S_head 128,
      // 7 % slower at S_head 64)
      stages(T_0{}, T_2{});
    } else {
      stages(T_0{}, T_1{});
      stages(T_1{}, T_2{});
    }
    __syncthreads();
  }
  bf16_t* out = dqkv + ((size_t)b * S_seq + key) * ld + head * D;
  if (dk_role) store_rows<D>(acc, out + h, lane, scale);
  else store_rows<D>(acc, out + 2 * h, lane, 1.0f);
  if (colpart) {
    // row (b, key block) of the partial column sums of [dK | dV], [S_mb * S_seq / 128][2 N_heads * D]
    float* red = reinterpret_cast<float*>(&QOs[0][0][0]);
    wave_colsum<D>(acc, dk_role ? scale : 1.0f, red + (size_t)w * 4 * (D / 2), lane);
    __syncthreads();
    if (tid < 2 * D) {
      const int dv = tid / D, d = tid - dv * D;  // dK from waves 4-7, dV from waves 0-3
      colpart[((size_t)b * (S_seq / WG_ROWS) + kblk) * 2 * h + dv * h + head * D + d] = colsum_of<D>(red, dv ? 0 : 4, 4, d);
    }
  }
}

template <int D>
bf_status fwd_d(int S_mb, int S_seq, int N_heads, int causal, const void* qkv, void* ctx, float* lse, hipStream_t st) {
  // the 256-query form when there are enough (head, block) pairs to give every compute unit one
  if (S_seq % 256 == 0 && (long)(S_seq / 256) * N_heads * S_mb >= 256) {
    const unsigned grid = (unsigned)(S_seq / 256) * N_heads * S_mb;
    attn_fwd_kernel<D, 256><<<grid, 512, 0, st>>>((const bf16_t*)qkv, (bf16_t*)ctx, lse, S_seq, N_heads, S_mb, causal, 1.0f / sqrtf((float)D));
  } else {
    const unsigned grid = (unsigned)(S_seq / 128) * N_heads * S_mb;
    attn_fwd_kernel<D, 128><<<grid, 256, 0, st>>>((const bf16_t*)qkv, (bf16_t*)ctx, lse, S_seq, N_heads, S_mb, causal, 1.0f / sqrtf((float)D));
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("attention_fwd_mfma launch failed: %s", hipGetErrorString(e)); return BF_EDEVICE; }
  return BF_OK;
}

template <int D>
bf_status bwd_d(int S_mb, int S_seq, int N_heads, int causal, const void* qkv, const void* ctx, const float* lse,
                const void* dctx, void* dqkv, float* delta, float* part, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)D);
  const unsigned grid = (unsigned)(S_seq / WG_ROWS) * N_heads * S_mb;
  // partial column sums: dQ's rows first, then those of [dK | dV]
  float* part_kv = part ? part + attention_bwd_mfma_part_q_rows(S_mb, S_seq) * (size_t)N_heads * D : nullptr;
  if (S_seq % 256 == 0)  // measured faster than the 128-query form also on grids that do not fill the chip
    attn_bwd_dq_kernel<D, 256><<<grid / 2, 512, 0, st>>>((const bf16_t*)qkv, (const bf16_t*)ctx, (const bf16_t*)dctx, lse, delta, (bf16_t*)dqkv, S_seq, N_heads, S_mb, causal, scale, part);
  else
    attn_bwd_dq_kernel<D, 128><<<grid, NTHR, 0, st>>>((const bf16_t*)qkv, (const bf16_t*)ctx, (const bf16_t*)dctx, lse, delta, (bf16_t*)dqkv, S_seq, N_heads, S_mb, causal, scale, part);
  attn_bwd_dkv_kernel<D><<<grid, NTHR_DKV, 0, st>>>((const bf16_t*)qkv, (const bf16_t*)dctx, lse, delta, (bf16_t*)dqkv, S_seq, N_heads, S_mb, causal, scale, part_kv);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_error("attention_bwd_mfma launch failed: %s", hipGetErrorString(e)); return BF_EDEVICE; }
  return BF_OK;
}

bool args_ok(int S_mb, int S_seq, int N_heads, int S_head, const void* a, const void* b2) {
  if (!attention_mfma_supported(S_seq, S_head)) { set_error("attention_mfma: needs S_head 64 or 128 and S_seq a multiple of 128"); return false; }
  if (S_mb < 1 || N_heads < 1 || S_mb > 65535 || N_heads > 65535) { set_error("attention_mfma: bad S_mb / N_heads"); return false; }
  if (((uintptr_t)a | (uintptr_t)b2) & 15) { set_error("attention_mfma: tensors must be 16-byte aligned"); return false; }
  return true;
}

}  // namespace

bool attention_mfma_supported(int S_seq, int S_head) {
  return (S_head == 64 || S_head == 128) && S_seq >= WG_ROWS && S_seq % WG_ROWS == 0;
}

bf_status attention_fwd_mfma(int S_mb, int S_seq, int N_heads, int S_head, int causal, const void* qkv, void* ctx,
                             float* lse, hipStream_t st) {
  if (!args_ok(S_mb, S_seq, N_heads, S_head, qkv, ctx)) return BF_EINVAL;
  if (S_head == 128) return fwd_d<128>(S_mb, S_seq, N_heads, causal, qkv, ctx, lse, st);
  return fwd_d<64>(S_mb, S_seq, N_heads, causal, qkv, ctx, lse, st);
}

// Rows of partial column sums the two backward kernels leave: one per (micro-batch sequence, query block) for dQ
// and one per (sequence, block of 128 keys) for [dK | dV].
size_t attention_bwd_mfma_part_q_rows(int S_mb, int S_seq) { return (size_t)S_mb * (S_seq / (S_seq % 256 == 0 ? 256 : WG_ROWS)); }
size_t attention_bwd_mfma_part_kv_rows(int S_mb, int S_seq) { return (size_t)S_mb * (S_seq / WG_ROWS); }

bf_status attention_bwd_mfma(int S_mb, int S_seq, int N_heads, int S_head, int causal, const void* qkv, const void* ctx,
                             const float* lse, const void* dctx, void* dqkv, float* delta, hipStream_t st, float* part) {
  if (!args_ok(S_mb, S_seq, N_heads, S_head, qkv, dqkv) || !args_ok(S_mb, S_seq, N_heads, S_head, ctx, dctx)) return BF_EINVAL;
  if (S_head == 128) return bwd_d<128>(S_mb, S_seq, N_heads, causal, qkv, ctx, lse, dctx, dqkv, delta, part, st);
  return bwd_d<64>(S_mb, S_seq, N_heads, causal, qkv, ctx, lse, dctx, dqkv, delta, part, st);
}

}  // namespace bf
