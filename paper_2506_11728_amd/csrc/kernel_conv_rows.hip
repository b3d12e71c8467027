// Convolution by lowering (paper Section 7.2: O = CONV(F, I) as a GEMM of dimensions
// (m, n, k) = (c_o, b h_o w_o, c_i h_f w_f) on the augmented matrix IM2COL(I)) for images
// whose channel count gives the tile kernels no aligned 16-byte runs to stream: the
// 3-channel first layer of a network, single-channel images.  The augmented matrix is
// never written.
//
// With k = (y, x, c), c fastest, the w_f * c_i bytes that one filter row y contributes
// to the row of an output position are one contiguous run of an image row:
//   bytes (ox*stride - pad) * c_i + r,  r = 0 .. w_f*c_i - 1,  of image row oy*stride + y - pad,
// and a byte of that run lies inside the image exactly when its position in the
// image row does (0 <= position < w_i * c_i), whatever its channel.  So a workgroup takes
// 128 consecutive output positions of one output row at a time (a tile), and
//   * its four loader waves stage the h_f image row segments the tile touches into LDS
//     (a few KB; zero where outside the image, every byte turned into the signed x - 128
//     on the way), into one of two stages, one tile ahead of the computation;
//   * its four compute waves build their operand fragments (32 positions x 32 k each)
//     from those segments: 16 consecutive k are at most two runs of bytes, fetched as two
//     16-byte LDS reads at whatever alignment and merged by a byte mask (filter rows
//     shorter than 16 bytes: byte by byte),
//   * multiply them with the filter fragments, laid out in LDS in register order once at
//     the workgroup's start (64 filters per workgroup, grid.y walks c_o),
//   * and write their 32 x 64 patches of O, starting the accumulators from the unsigned
//     correction 128 * sum_k F(o, k) (overwrite / accumulate, optional scale to float).
// A workgroup walks several tiles (stride gridDim.x), so the filter fragments are built
// once, and the split into loader and compute waves keeps the image loads and the waits
// for them out of the way of the stores of O.  Bound by the write of O in principle;
// measured, instruction issue of the fragment building and the write-back still shows.
#include "epilogue.h"
#include "lds_layout.h"
#include "mip_internal.h"

namespace mip {

namespace {

constexpr int TP = 128;  // output positions per tile: 32 per wave
constexpr int TN = 64;   // filters per workgroup: two 32-wide blocks per wave
constexpr int MAX_LDS = 64 * 1024;
// after the image stage and the filter fragments: 64 column sums, 64 accumulator start
// values, the table of runs (at most 32 k steps), one write-back patch per wave
constexpr int FIXED_LDS = 256 + 256 + 1024 + 4 * STORE_PATCH_BYTES;
constexpr int NTHREADS_ROWS = 512;  // four compute waves and four loader waves
constexpr int NCOMPUTE = 256;
constexpr int STAGE_ROWS = 8;  // image words (of as many segments) a loader thread has in flight

struct RowsParams {
  ConvGeom G;
  int hf;
  int k;              // hf * wf * ci
  int ksteps;         // k in steps of 32, rounded up
  int n;              // c_o
  int tiles_per_row;  // tiles along one output row
  int64_t tiles;      // b * ho * tiles_per_row
  int row_bytes;      // pitch of one staged image row segment (multiple of 4)
  int stage_bytes;    // hf segments, rounded up to 16
  const uint8_t *I;
  const uint8_t *F;
  int32_t *O;
  int accumulate, out_float;
  float scale;
};

struct __attribute__((packed, aligned(1))) unaligned_word { uint32_t w; };

// store_blocks_via_lds of the shared epilogue for a patch of which only the first `rows`
// rows exist: one 32 x 32 block at a time through the wave's LDS patch, whole 128-byte
// lines of O per store instruction.
__device__ __forceinline__ void store_rows_via_lds(const v16i (&acc)[1][2], int32_t *C, int ldc,
                                                   int rows, bool accumulate, int lane,
                                                   int32_t *patch, const Finish fin) {
  // the piece of block j this lane handles in pass t: 4 words of row t * 8 + lane / 8
  // (a 32 x 64 patch of O spans fewer than 2^31 words: a uniform base and a 32-bit offset)
  const int r0 = lane >> 3, c0 = (lane & 7) * 4;
  auto piece = [&](int j, int t) {
    return reinterpret_cast<v4i_dword_aligned *>(C + (uint32_t)((t * 8 + r0) * ldc + j * 32 + c0));
  };
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    // an accumulating call has the old words of the block in flight before its first store
    v4i old[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      old[t] = v4i{0, 0, 0, 0};
      if (accumulate && t * 8 + r0 < rows) old[t] = __builtin_nontemporal_load(piece(j, t));
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      v4i val = {acc[0][j][4 * q], acc[0][j][4 * q + 1], acc[0][j][4 * q + 2], acc[0][j][4 * q + 3]};
      *reinterpret_cast<v4i *>(patch + (lane & 31) * 36 + 8 * q + 4 * (lane >> 5)) = val;
    }
    // same wave wrote and reads: LDS operations of a wave complete in order
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      v4i val = *reinterpret_cast<const v4i *>(patch + (t * 8 + r0) * 36 + c0);
      if (t * 8 + r0 < rows) {
#pragma unroll
        for (int e = 0; e < 4; ++e) val[e] = fin(val[e], old[t][e], accumulate);
        __builtin_nontemporal_store(val, piece(j, t));
      }
    }
  }
}

// TO_FLOAT, ACCUMULATE: what the write-back does, fixed at compile time.
template <bool TO_FLOAT, bool ACCUMULATE>
__global__ __launch_bounds__(NTHREADS_ROWS) void conv_rows_kernel(RowsParams P) {
  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  // two image stages, the filter fragments, then the small tables and the write-back patches
  v4i *ffrag = reinterpret_cast<v4i *>(smem + 2 * P.stage_bytes);  // [ksteps][2][64 lanes]
  int *colsum = reinterpret_cast<int *>(smem + 2 * P.stage_bytes + P.ksteps * 2048);  // [64]
  v4i *start = reinterpret_cast<v4i *>(colsum + 64);  // [2 lane halves][2 blocks][4]: accumulator start values
  v4i *runs = start + 16;  // [ksteps][2 lane halves]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int32_t *patch = reinterpret_cast<int32_t *>(runs + 64) + (wave & 3) * STORE_PATCH_WORDS;
  const int n0 = blockIdx.y * TN;
  const int wfci = P.G.wf * P.G.ci;
  const int row_len = P.G.wi * P.G.ci;  // bytes of one image row

  // filter fragments in register order: lane l of block j holds filter n0 + 32 j + l % 32,
  // k = 32 ks + 16 (l / 32) .. + 15; zero past k and past the last filter
  for (int slot = tid; slot < P.ksteps * 128; slot += NTHREADS_ROWS) {
    const int l = slot & 63, j = (slot >> 6) & 1, ks = slot >> 7;
    const int co = n0 + 32 * j + (l & 31);
    const int kk0 = 32 * ks + 16 * (l >> 5);
    // every load unconditional (clamped into the filter tensor, zeroed afterwards), so that
    // they are all in flight together
    const uint8_t *row = P.F + (int64_t)(co < P.n ? co : P.n - 1) * P.k;
    v4i f = {0, 0, 0, 0};
    if (kk0 + 16 <= P.k) {
      f = load16(row + kk0);
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int kk = kk0 + e;
        const uint32_t x = row[kk < P.k ? kk : P.k - 1];
        f[e >> 2] |= (int)((kk < P.k ? x : 0u) << (8 * (e & 3)));
      }
    }
    if (co >= P.n) f = v4i{0, 0, 0, 0};
    ffrag[slot] = f;
  }
  __syncthreads();
  // The image bytes are staged as x - 128, so every sum lacks 128 * sum_k F(o, k) (exact
  // modulo 2^32): the accumulators start from that instead of zero.  Laid out as the
  // registers want it: lane half h, block j, register v stands for filter 32 j + 8 (v / 4)
  // + 4 h + v % 4.
  if (wave == 0) {
    int sumB[2] = {0, 0};  // this lane's half of sum_k F(o, k) for its two filters
    for (int ks = 0; ks < P.ksteps; ++ks)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const v4i f = ffrag[(ks * 2 + j) * 64 + lane];
#pragma unroll
        for (int r = 0; r < 4; ++r) sumB[j] = __builtin_amdgcn_sdot4(f[r], 0x01010101, sumB[j], false);
      }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int total = sumB[j] + __shfl_xor(sumB[j], 32);
      if (lane < 32) colsum[32 * j + lane] = total;
    }
  }
  __syncthreads();
  if (tid < 64) {
    const int h = tid >> 5, j = (tid >> 4) & 1, v = tid & 15;
    reinterpret_cast<int *>(start)[tid] = 128 * colsum[32 * j + 8 * (v >> 2) + 4 * h + (v & 3)];
  }
  // where the 16 bytes k = 32 ks + 16 h .. + 15 of a position start in the stage (first run:
  // offset and length; second run: offset less the first run's length, relative to the first)
  if (tid >= 64 && tid < 64 + 2 * P.ksteps && wfci >= 16) {
    const int e = tid - 64, kk0 = 16 * e;  // e = 2 ks + h
    v4i run = {0, 16, 0, 0};
    if (kk0 < P.k) {
      const int y0 = kk0 / wfci, r = kk0 - y0 * wfci;
      run[0] = y0 * P.row_bytes + r;
      run[1] = wfci - r;
      run[2] = run[1] < 16 && y0 + 1 < P.hf ? P.row_bytes - wfci : 0;
    }
    runs[e] = run;
  }
  // (the barrier before the tile loop publishes the start values and the runs)

  const Finish fin = {P.scale, TO_FLOAT ? 1 : 0};

  struct Tile {
    int64_t orow;  // g * ho + oy
    int ox0;       // first output column
    int iy0;       // image row of filter row 0
    int pos0;      // image-row position of staged byte 0
    int words;     // words per staged segment
    const uint8_t *image;
  };
  auto tile_at = [&](int t) {  // (fewer tiles than output positions, and those fit 31 bits)
    Tile T;
    const int orow = t / P.tiles_per_row;
    T.orow = orow;
    T.ox0 = (t - orow * P.tiles_per_row) * TP;
    const int g = orow / P.G.ho, oy = orow - g * P.G.ho;
    T.iy0 = oy * P.G.stride - P.G.pad;
    T.pos0 = (T.ox0 * P.G.stride - P.G.pad) * P.G.ci;
    T.image = P.I + (int64_t)g * P.G.hi * row_len;
    // only the bytes that positions inside the output row touch are staged; the fragments
    // of the positions past its end read whatever LDS holds and are never stored
    const int live = P.G.wo - T.ox0 < TP ? P.G.wo - T.ox0 : TP;
    T.words = (((live - 1) * P.G.stride + P.G.wf) * P.G.ci + 3) / 4;
    return T;
  };

  // A loader thread's work for one tile: its share of the hf image row segments into `img`,
  // zero where outside the image, every byte x turned into the signed x - 128.  It takes
  // one word position of STAGE_ROWS segments at a time: all loads first, every one
  // unconditional (row and position clamped into the image) so that they are in flight
  // together, then the LDS stores.  A word that straddles an end of the image row is the
  // clamped word shifted, zeros moving in (the host sends no image row shorter than a word).
  auto stage_tile = [&](const Tile &T, uint8_t *img) {
    for (int d = tid - NCOMPUTE; d < T.words; d += NTHREADS_ROWS - NCOMPUTE) {
      const int pos = T.pos0 + 4 * d;
      const int pos_in = pos < 0 ? 0 : (pos + 3 < row_len ? pos : row_len - 4);
      const int shift = pos - pos_in;  // bytes: > 0 past the right end, < 0 before the left end
      const int right = shift > 0 ? (shift < 4 ? 8 * shift : 32) : 0;
      const int left = shift < 0 ? (shift > -4 ? -8 * shift : 32) : 0;
      for (int y0 = 0; y0 < P.hf; y0 += STAGE_ROWS) {
        uint32_t w[STAGE_ROWS];
#pragma unroll
        for (int u = 0; u < STAGE_ROWS; ++u) {
          int iy = T.iy0 + y0 + u;
          iy = iy < 0 ? 0 : (iy >= P.G.hi ? P.G.hi - 1 : iy);
          // (an image is shorter than 2^31 bytes: a uniform base and a 32-bit offset)
          w[u] = reinterpret_cast<const unaligned_word *>(T.image + (uint32_t)(iy * row_len + pos_in))->w;
        }
#pragma unroll
        for (int u = 0; u < STAGE_ROWS; ++u) {
          const int y = y0 + u, iy = T.iy0 + y;
          // 64-bit shifts: a distance of 32 clears the word
          uint32_t v = (uint32_t)(((uint64_t)w[u] >> right) << left);
          v = iy >= 0 && iy < P.G.hi ? v : 0u;
          if (y < P.hf) *reinterpret_cast<uint32_t *>(img + y * P.row_bytes + 4 * d) = v ^ 0x80808080u;
        }
      }
    }
  };

  // A compute wave's work for one tile: 32 positions x 64 filters.
  auto compute_tile = [&](const Tile &T, const uint8_t *img) {
    v16i acc[1][2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const v4i c = start[((lane >> 5) * 2 + j) * 4 + q];
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[0][j][4 * q + e] = c[e];
      }
    const int lane_base = (wave * 32 + (lane & 31)) * P.G.stride * P.G.ci;
    // 16 consecutive k of this lane's position, starting at kk0.  Bytes at k and beyond meet
    // zeros in the filter fragments, so they may be anything: only the addresses matter.
    // Filter rows of 16 bytes or more: at most two runs, each fetched as 16 bytes at whatever
    // alignment (reads may run up to 15 bytes past the stage, into what follows it in LDS),
    // merged by a byte mask.
    auto gather_runs = [&](int ks) {
      const v4i run = runs[2 * ks + (lane >> 5)];
      const int off1 = run[0] + lane_base, n1 = run[1], off2 = off1 + run[2];
      const v4i v1 = load16(img + off1), v2 = load16(img + off2);
      v4i fa;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const int cnt = n1 - 4 * d;  // bytes of this word that still belong to the first run
        const uint32_t mask = cnt >= 4 ? 0xFFFFFFFFu : (cnt <= 0 ? 0u : (1u << (8 * cnt)) - 1u);
        fa[d] = (int)(((uint32_t)v1[d] & mask) | ((uint32_t)v2[d] & ~mask));
      }
      return fa;
    };
    // any filter row length: byte by byte
    auto gather_bytes = [&](int kk0) {
      const int y0 = kk0 / wfci;
      int r = kk0 - y0 * wfci;
      int off = y0 * P.row_bytes + lane_base + r;  // inside the stage while kk < k
      v4i fa = {0, 0, 0, 0};
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const uint32_t x = img[kk0 + e < P.k ? off : 0];
        fa[e >> 2] |= (int)(x << (8 * (e & 3)));
        ++r;
        ++off;
        if (r == wfci) {  // next filter row: next staged segment, same position
          r = 0;
          off += P.row_bytes - wfci;
        }
      }
      return fa;
    };
    for (int ks = 0; ks < P.ksteps; ++ks) {
      const int kk0 = 32 * ks + 16 * (lane >> 5);
      const v4i fa = wfci >= 16 ? gather_runs(ks) : gather_bytes(kk0);
      const v4i f0 = ffrag[(ks * 2) * 64 + lane], f1 = ffrag[(ks * 2 + 1) * 64 + lane];
      acc[0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f0, fa, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(f1, fa, acc[0][1], 0, 0, 0);
    }

    const int oxw = T.ox0 + wave * 32;  // wave-uniform
    if (oxw < P.G.wo) {
      int32_t *C = P.O + (T.orow * P.G.wo + oxw) * (int64_t)P.n + n0;
      const int rows = P.G.wo - oxw < 32 ? P.G.wo - oxw : 32;
      if (P.out_float == 2) {  // int8 output (overwrite only): O is a tensor of bytes
        int8_t *Q = reinterpret_cast<int8_t *>(P.O) + (T.orow * P.G.wo + oxw) * (int64_t)P.n + n0;
        store_blocks_q8<1, 2>(acc, Q, P.n, rows, P.n - n0, lane, P.scale);
      } else if (P.n - n0 >= TN)  // all 64 filters: full lines through the wave's LDS patch
        store_rows_via_lds(acc, C, P.n, rows, ACCUMULATE, lane, patch, fin);
      else
        store_blocks<1, 2, false>(acc, C, P.n, rows, P.n - n0, ACCUMULATE, lane, fin);
    }
  };

  // Four compute waves and four loader waves (two waves on every SIMD).  While the compute
  // waves work on one stage and write their patch of O, the loader waves fill the other
  // stage with the next tile: their loads, and the waits for them, never stand behind
  // stores (a wave's memory counter is its own, and stores count in it), and the compute
  // waves never wait for loads.
  // The two kinds of waves run loops of their own, with the same number of barriers (whole
  // waves take either branch, and a barrier counts waves wherever they wait): so each loop
  // is scheduled, and its memory waits are placed, for what that kind of wave does.
  // The barrier is issued as the bare instruction with explicit fences, not as __syncthreads():
  // the two loops sit in branches that whole waves take differently, which a convergent
  // workgroup barrier of the language does not allow for.  Both kinds of wave execute exactly
  // 1 + trips barriers, trips = the number of tiles t = blockIdx.x, blockIdx.x + step, ... below
  // ntiles, the same expression in both loops.
  auto role_barrier = []() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  };
  const int ntiles = (int)P.tiles, step = (int)gridDim.x;
  if (wave >= 4) {
    stage_tile(tile_at(blockIdx.x), smem);  // the host launches no more workgroups than tiles
    role_barrier();
    int cur = 0;
    for (int t = blockIdx.x; t < ntiles; t += step) {
      if (ntiles - t > step) stage_tile(tile_at(t + step), smem + (cur ^ 1) * P.stage_bytes);
      role_barrier();  // the next stage is filled, this one is free
      cur ^= 1;
    }
  } else {
    role_barrier();
    int cur = 0;
    for (int t = blockIdx.x; t < ntiles; t += step) {
      compute_tile(tile_at(t), smem + cur * P.stage_bytes);
      role_barrier();
      cur ^= 1;
    }
  }
}

bool fill_params(const Problem &p, RowsParams *out) {
  if (!p.conv || !p.a_unsigned || p.b_unsigned || p.batch != 1) return false;
  if (p.b_sk != 1 || p.b_sn != p.k || p.m < 1 || p.n < 1 || p.k < 1) return false;
  if (p.m >= ((int64_t)1 << 30)) return false;  // tile numbers are 32-bit in the kernel
  const ConvGeom &G = *p.conv;
  const int64_t wfci = (int64_t)G.wf * G.ci;
  if (p.k % wfci != 0 || p.k > 4096) return false;
  const int64_t hf = p.k / wfci;
  const int64_t seg = ((int64_t)(TP - 1) * G.stride + G.wf) * G.ci;  // bytes of one staged segment
  const int64_t row_bytes = (seg + 3) / 4 * 4;
  const int64_t stage = (hf * row_bytes + 15) / 16 * 16;
  const int64_t ksteps = (p.k + 31) / 32;
  if (ksteps > 32 || 2 * stage + ksteps * 2048 + FIXED_LDS > MAX_LDS) return false;
  // image-row positions are formed in 32 bits, also for the tile that overhangs the row
  if (((int64_t)G.wo + TP) * G.stride * G.ci + (int64_t)G.pad * G.ci >= ((int64_t)1 << 30)) return false;
  if ((int64_t)G.wi * G.ci >= ((int64_t)1 << 30) || (int64_t)G.wi * G.ci < 4) return false;
  if ((p.n + TN - 1) / TN > 65535) return false;
  RowsParams P;
  P.G = G;
  P.hf = (int)hf;
  P.k = (int)p.k;
  P.ksteps = (int)ksteps;
  P.n = (int)p.n;
  P.tiles_per_row = (G.wo + TP - 1) / TP;
  P.tiles = p.m / G.wo * P.tiles_per_row;  // m = b * ho * wo
  P.row_bytes = (int)row_bytes;
  P.stage_bytes = (int)stage;
  P.I = static_cast<const uint8_t *>(p.A);
  P.F = static_cast<const uint8_t *>(p.B);
  P.O = p.C;
  P.accumulate = p.accumulate;
  P.out_float = p.out_float;
  P.scale = p.scale;
  *out = P;
  return true;
}

}  // namespace

bool conv_rows_eligible(const Problem &p) {
  RowsParams P;
  return fill_params(p, &P);
}

hipError_t launch_conv_rows(const Problem &p, hipStream_t s) {
  RowsParams P;
  if (!fill_params(p, &P)) return hipErrorInvalidValue;
  // at most as many workgroups as the 256 compute units hold at once (two each, by
  // registers), each with the same number of tiles
  int64_t wgs = P.tiles < 512 ? P.tiles : 512;
  const int64_t per = (P.tiles + wgs - 1) / wgs;
  wgs = (P.tiles + per - 1) / per;
  dim3 grid((unsigned)wgs, (unsigned)((P.n + TN - 1) / TN), 1);
  const size_t lds = 2 * (size_t)P.stage_bytes + (size_t)P.ksteps * 2048 + FIXED_LDS;
  const dim3 block(NTHREADS_ROWS);
  if (P.out_float == 2) {  // (the integer instance: its int8 branch is taken at run time)
    if (P.accumulate) return hipErrorInvalidValue;
    hipLaunchKernelGGL((conv_rows_kernel<false, false>), grid, block, lds, s, P);
  } else if (P.out_float && P.accumulate) hipLaunchKernelGGL((conv_rows_kernel<true, true>), grid, block, lds, s, P);
  else if (P.out_float) hipLaunchKernelGGL((conv_rows_kernel<true, false>), grid, block, lds, s, P);
  else if (P.accumulate) hipLaunchKernelGGL((conv_rows_kernel<false, true>), grid, block, lds, s, P);
  else hipLaunchKernelGGL((conv_rows_kernel<false, false>), grid, block, lds, s, P);
  return hipGetLastError();
}

}  // namespace mip
