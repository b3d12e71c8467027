// The skinny-m kernel (m <= 64: a handful of tokens against a weight matrix).
//
// Such a GEMM is a stream of B through the chip, once: it is bound by memory, not
// by the matrix cores, and there are too few C tiles to give every compute unit
// one.  The tiled kernels answer that by splitting k over workgroups, which costs
// a zero-fill launch and atomic traffic on C.  Here a workgroup instead owns a
// narrow slab of B, 16, 32 or 64 columns wide and all of k deep, so that n / 16
// workgroups exist and nothing is shared between them: one launch, plain stores.
// Inside the workgroup the four waves split k (wave w takes the 64-deep steps
// w, w + 4, ...), each wave streams its steps through a private ring in LDS with
// direct loads and no workgroup barrier, and the four partial sums meet in LDS at
// the end.  The micro-kernel is v_mfma_i32_16x16x64_i8: 16 rows of A are all a
// skinny problem has, and 16 columns keep the slab narrow.
//
// Fragment layout of that instruction (as for the 32 x 32 x 32 form): lane l
// supplies, for row (A) or column (B) l % 16, the 16 bytes k = 16 * (l / 16) ..
// + 15 of the 64-deep step; in the result lane l holds column l % 16, register v
// holds row 4 * (l / 16) + v.
//
// Preconditions, checked on the host (slab_eligible): 1 <= m <= 64, A stored with
// k contiguous, n a multiple of 16, k a multiple of 64, 16-byte aligned operand
// bases and leading dimensions.
#include "dma_common.h"

namespace mip {

namespace {

constexpr int DA = 4;  // steps of A in flight per wave (A is small: cache latency)
// steps of B in flight per wave (memory latency): 8 KB of a narrow slab, 16 KB of a 64-column one
constexpr int steps_of_b_in_flight(int nt) { return nt >= 4 ? 4 : 8; }

struct SlabParams {
  const uint8_t *A, *B;
  int32_t *C;
  int64_t lda, ldb, ldc;
  int m;
  int nsteps;      // k / 64
  int tiles;       // n / (16 * NT)
  int accumulate;  // C += instead of C =
  int out_float;   // dequantised output: float(sum) * scale
  float scale;
};

// A pointer that is the same in every lane, said so that it stays in SGPRs (the
// direct loads need a scalar base).
__device__ __forceinline__ const uint8_t *wave_uniform(const uint8_t *p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
}

template <int N>
__device__ __forceinline__ void loads_landed() {  // all but the N newest direct loads
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// MT: row blocks of 16 (m <= 16 * MT).  NT: column blocks of 16 per workgroup.
// B_KC: B stored with k contiguous (column-major).  UNS: 0 both signed, 1 A
// unsigned, 2 B unsigned.
template <int MT, int NT, bool B_KC, int UNS>
__global__ __launch_bounds__(NTHREADS) void slab_kernel(SlabParams P) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  constexpr int DB = steps_of_b_in_flight(NT);
  constexpr int B_STEP = NT * 1024, A_STEP = MT * 1024;  // bytes of one 64-deep step
  constexpr int WAVE_BYTES = DB * B_STEP + DA * A_STEP;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // consecutive workgroup ids sit on different XCDs: give each XCD a contiguous run
  // of slabs, so that neighbours, which share cache lines of a row-major B, share an L2
  const int per_xcd = (P.tiles + 7) / 8;
  const int tile = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if ((int)(blockIdx.x / 8) >= per_xcd || tile >= P.tiles) return;
  const int64_t n0 = (int64_t)tile * 16 * NT;

  uint8_t *ringB = smem + wave * WAVE_BYTES;
  uint8_t *ringA = ringB + DB * B_STEP;
  const uint32_t ldsB = lds_address(ringB), ldsA = lds_address(ringA);

  // Which 16 bytes each lane fetches.  A and a k-contiguous B arrive in fragment
  // order (lane l: row or column l % 16, k chunk l / 16), so the MFMA operand is
  // one linear 16-byte read.  A row-major B arrives as 64 k rows of 16 * NT bytes
  // and is turned by the transposing LDS read.
  uint32_t offA[MT], offB[NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int row = 16 * mt + (lane & 15);
    row = row < P.m ? row : P.m - 1;  // rows past m repeat the last one and are never stored
    offA[mt] = (uint32_t)(row * P.lda + 16 * (lane >> 4));
  }
#pragma unroll
  for (int q = 0; q < NT; ++q)
    offB[q] = B_KC ? (uint32_t)((16 * q + (lane & 15)) * P.ldb + 16 * (lane >> 4))
                   : (uint32_t)((q * (64 / NT) + lane / NT) * P.ldb + 16 * (lane % NT));
  const uint8_t *baseB = B_KC ? P.B + n0 * P.ldb : P.B + n0;
  const int64_t strideB = B_KC ? 64 : 64 * P.ldb;  // one step further down k

  const int cnt = (P.nsteps + 3 - wave) / 4;  // steps wave, wave + 4, ... below nsteps
  auto issueB = [&](int i) __attribute__((always_inline)) {
    if (i < cnt) {
      const uint8_t *g = wave_uniform(baseB + (int64_t)(wave + 4 * i) * strideB);
      const uint32_t slot = ldsB + (i % DB) * B_STEP;
#pragma unroll
      for (int q = 0; q < NT; ++q) dma16(offB[q], g, slot + q * 1024);
    }
  };
  auto issueA = [&](int i) __attribute__((always_inline)) {
    if (i < cnt) {
      const uint8_t *g = wave_uniform(P.A + (int64_t)(wave + 4 * i) * 64);
      const uint32_t slot = ldsA + (i % DA) * A_STEP;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) dma16(offA[mt], g, slot + mt * 1024);
    }
  };

  v4i acc[MT][NT];
  int sumA[MT], sumB[NT];  // k sums of the signed operand (unsigned-operand correction)
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    sumA[mt] = 0;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = v4i{0, 0, 0, 0};
  }
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) sumB[nt] = 0;

  // The loads go out in one fixed interleaved order, B of step j + DB then A of
  // step j + DA, from j = -DB on.  Loads complete in order, so when step j is to
  // be used, everything issued after its A fragment, i.e. what the DA - 1
  // iterations since then sent out, may still be in flight and nothing else.
  constexpr int NEWER = (DA - 1) * (NT + MT);
  for (int j = -DB; j < 0; ++j) {
    issueB(j + DB);
    if (j + DA >= 0) issueA(j + DA);
  }
  for (int j = 0; j < cnt; ++j) {
    // near the end fewer loads follow: wait for all of them
    if (j + DB <= cnt) loads_landed<NEWER>();
    else loads_landed<0>();

    const uint8_t *sa = ringA + (j % DA) * A_STEP;
    const uint8_t *sb = ringB + (j % DB) * B_STEP;
    v4i fa[MT], fb[NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      fa[mt] = *reinterpret_cast<const v4i *>(sa + mt * 1024 + 16 * lane);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      if (B_KC) {
        fb[nt] = *reinterpret_cast<const v4i *>(sb + nt * 1024 + 16 * lane);
      } else {
        // transposing read: in each group of 16 lanes, lane 2t + h names half h of the
        // 16-byte row t and lane i receives byte i of rows 0..7
        const int krow = 16 * (lane >> 4) + ((lane & 15) >> 1);
#pragma unroll
        for (int r = 0; r < 2; ++r) {
          const int off = (krow + 8 * r) * (16 * NT) + 16 * nt + 8 * (lane & 1);
          v2i h = __builtin_amdgcn_ds_read_tr8_b64_v2i32(LDS_PTR(v2i, sb + off));
          fb[nt][2 * r] = h[0];
          fb[nt][2 * r + 1] = h[1];
        }
      }
    }
    if (UNS == 1) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) fa[mt] ^= (int)0x80808080u;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          sumB[nt] = __builtin_amdgcn_sdot4(fb[nt][r], 0x01010101, sumB[nt], false);
    }
    if (UNS == 2) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) fb[nt] ^= (int)0x80808080u;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          sumA[mt] = __builtin_amdgcn_sdot4(fa[mt][r], 0x01010101, sumA[mt], false);
    }
    // the fragments are in registers before the slots they came from are refilled
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[mt], fb[nt], acc[mt][nt], 0, 0, 0);
    issueB(j + DB);
    issueA(j + DA);
  }
  loads_landed<0>();

  // unsigned operand: sum (x - 128) y + 128 sum y, each wave for its own share of k
  if (UNS == 1) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      int t = sumB[nt];
      t += __shfl_xor(t, 16);
      t += __shfl_xor(t, 32);  // every lane: the sum of its own column l % 16
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) acc[mt][nt] += 128 * t;
    }
  }
  if (UNS == 2) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      int t = sumA[mt];
      t += __shfl_xor(t, 16);
      t += __shfl_xor(t, 32);  // lane l: the sum of row l % 16
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int c = 128 * __shfl(t, 4 * (lane >> 4) + v);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt][v] += c;
      }
    }
  }

  // the four partial sums meet in LDS, over the rings, once every wave is done with them
  __syncthreads();
  v4i *red = reinterpret_cast<v4i *>(smem);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) red[((wave * MT + mt) * NT + nt) * 64 + lane] = acc[mt][nt];
  __syncthreads();
  const Finish fin{P.scale, P.out_float};
  for (int b = wave; b < MT * NT; b += 4) {
    const int mt = b / NT, nt = b % NT;
    v4i s = red[(mt * NT + nt) * 64 + lane];
#pragma unroll
    for (int w = 1; w < 4; ++w) s += red[((w * MT + mt) * NT + nt) * 64 + lane];
    int32_t *c = P.C + n0 + 16 * nt + (lane & 15);
    // (an accumulating call reads its four old words before the first store, not one behind each)
    int old[4] = {0, 0, 0, 0};
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = 16 * mt + 4 * (lane >> 4) + v;
      if (P.accumulate && row < P.m) old[v] = c[row * P.ldc];
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int row = 16 * mt + 4 * (lane >> 4) + v;
      if (row < P.m) c[row * P.ldc] = fin(s[v], old[v], P.accumulate != 0);
    }
  }
}

template <int MT, int NT>
void (*pick(bool b_kc, int uns))(SlabParams) {
  if (b_kc) return uns == 0 ? slab_kernel<MT, NT, true, 0>
                            : (uns == 1 ? slab_kernel<MT, NT, true, 1> : slab_kernel<MT, NT, true, 2>);
  return uns == 0 ? slab_kernel<MT, NT, false, 0>
                  : (uns == 1 ? slab_kernel<MT, NT, false, 1> : slab_kernel<MT, NT, false, 2>);
}

}  // namespace

bool slab_eligible(const Problem &p, int nt) {
  if (p.conv || p.batch != 1 || p.m < 1 || p.m > 64 || p.a_sk != 1) return false;
  if (p.out_float == 2) return false;  // (no int8 write-back here)
  if (nt != 1 && nt != 2 && nt != 4) return false;
  if (p.n % (16 * nt) || p.k % 64 || p.k < 64) return false;
  if (p.b_sk != 1 && p.b_sn != 1) return false;
  const int64_t lda = p.a_sm, ldb = p.b_sk == 1 ? p.b_sn : p.b_sk;
  if ((p.m > 1 && lda % 16) || ldb % 16) return false;  // a single row of A has no stride
  if (reinterpret_cast<uintptr_t>(p.A) % 16 || reinterpret_cast<uintptr_t>(p.B) % 16) return false;
  if ((p.m > 1 && 64 * lda >= ((int64_t)1 << 31)) || 64 * ldb >= ((int64_t)1 << 31)) return false;
  if (p.n / (16 * nt) > ((int64_t)1 << 30)) return false;
  return true;
}

hipError_t launch_slab(const Problem &p, int nt, hipStream_t s) {
  SlabParams P;
  P.A = static_cast<const uint8_t *>(p.A);
  P.B = static_cast<const uint8_t *>(p.B);
  P.C = p.C;
  P.lda = p.a_sm;
  const bool b_kc = p.b_sk == 1;
  P.ldb = b_kc ? p.b_sn : p.b_sk;
  P.ldc = p.ldc;
  P.m = (int)p.m;
  P.nsteps = (int)(p.k / 64);
  P.tiles = (int)(p.n / (16 * nt));
  P.accumulate = p.accumulate;
  P.out_float = p.out_float;
  P.scale = p.scale;
  const int uns = p.a_unsigned ? 1 : (p.b_unsigned ? 2 : 0);
  const int mt = p.m <= 16 ? 1 : (p.m <= 32 ? 2 : 4);
  void (*kern)(SlabParams) = nullptr;
  if (nt == 1) kern = mt == 1 ? pick<1, 1>(b_kc, uns) : (mt == 2 ? pick<2, 1>(b_kc, uns) : pick<4, 1>(b_kc, uns));
  else if (nt == 2) kern = mt == 1 ? pick<1, 2>(b_kc, uns) : (mt == 2 ? pick<2, 2>(b_kc, uns) : pick<4, 2>(b_kc, uns));
  else kern = mt == 1 ? pick<1, 4>(b_kc, uns) : (mt == 2 ? pick<2, 4>(b_kc, uns) : pick<4, 4>(b_kc, uns));
  const size_t lds = (size_t)4 * (steps_of_b_in_flight(nt) * nt + DA * mt) * 1024;
  {
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds);
    if (e != hipSuccess) return e;
  }
  dim3 grid((unsigned)(((P.tiles + 7) / 8) * 8));
  hipLaunchKernelGGL(kern, grid, dim3(NTHREADS), lds, s, P);
  return hipGetLastError();
}

}  // namespace mip
