// LDS layouts of one staged operand block and the fragment reads that feed
// v_mfma_i32_32x32x32_i8, shared by the MFMA kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mip {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
struct __attribute__((packed, aligned(1))) unaligned_v4i { v4i v; };

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr int BK = 64;        // k per staged block
constexpr int NTHREADS = 256; // 4 waves, arranged 2 x 2 over the tile

// 16 bytes, of which only the first nvalid are read; the rest are zero.
__device__ __forceinline__ v4i load16_partial(const uint8_t *p, int nvalid) {
  v4i r = {0, 0, 0, 0};
#pragma unroll
  for (int b = 0; b < 16; ++b) {
    uint32_t x = b < nvalid ? p[b] : 0u;
    r[b >> 2] |= (int)(x << (8 * (b & 3)));
  }
  return r;
}

__device__ __forceinline__ v4i load16(const uint8_t *p) {
  return reinterpret_cast<const unaligned_v4i *>(p)->v;
}

// One operand block in LDS.
// KD is the depth of the block along k (64 or 128).
//   KC (k contiguous in memory: row-major A, column-major B):
//     R rows of KD bytes; 16-byte chunk c of row r sits at r*KD + 16*(c ^ kswz(r)).
//   strided (the index runs contiguously: column-major A, row-major B):
//     KD k-rows of R bytes; chunk c of k-row q sits at q*R + 16*(c ^ swz(q)).
// Both XOR patterns spread the 16 lanes of one LDS access over all banks
// (no bank conflicts measured).
template <int R, bool KC, int KD = BK>
struct Stage {
  static constexpr int CHUNKS = R * KD / 16;
  static constexpr int PER_THREAD = CHUNKS / NTHREADS;
  static constexpr int ROW_CHUNKS = R / 16;  // strided: chunks per k-row
  static constexpr int K_CHUNKS = KD / 16;   // KC: chunks per row

  // rows 256 bytes apart share banks: rotate their chunks against each other
  __device__ static __forceinline__ int kswz(int r) { return (r / (256 / KD)) % K_CHUNKS; }

  __device__ static __forceinline__ int swz(int q) { return 2 * ((q / (256 / R)) % (R / 32)); }

  // chunk handled by this thread: (row, chunk-in-row) for KC, (k-row, chunk) for strided
  __device__ static __forceinline__ void chunk_of(int i, int tid, int &a, int &c) {
    int q = tid + NTHREADS * i;
    if (KC) { a = q / K_CHUNKS; c = q % K_CHUNKS; }
    else { a = q / ROW_CHUNKS; c = q % ROW_CHUNKS; }
  }

  __device__ static __forceinline__ int lds_offset(int a, int c) {
    if (KC) return a * KD + ((c ^ kswz(a)) << 4);
    return a * R + ((c ^ swz(a)) << 4);
  }

  // Global -> registers.  r0: first row (m or n index) of the block, k0: first k.
  // ext: number of valid rows, kext: number of valid k.  sr / sk: byte strides.
  template <bool CHECKED>
  __device__ static __forceinline__ void load(v4i (&reg)[PER_THREAD], const uint8_t *base,
                                             int64_t sr, int64_t sk, int64_t r0, int64_t k0,
                                             int64_t ext, int64_t kext, int tid, int flip) {
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      int a, c;
      chunk_of(i, tid, a, c);
      v4i v;
      if (KC) {
        int64_t row = r0 + a, kk = k0 + c * 16;
        if (!CHECKED) {
          v = load16(base + row * sr + kk);
        } else {
          if (row > ext - 1) row = ext - 1;  // rows past the edge: any valid row, never stored
          int64_t left = kext - kk;
          const uint8_t *p = base + row * sr + kk;
          if (left >= 16) v = load16(p);
          else v = load16_partial(p, left > 0 ? (int)left : 0);
        }
      } else {
        int64_t kq = k0 + a, col = r0 + c * 16;
        if (!CHECKED) {
          v = load16(base + kq * sk + col);
        } else {
          int64_t left = kq < kext ? ext - col : 0;
          const uint8_t *p = base + kq * sk + col;
          if (left >= 16) v = load16(p);
          else v = load16_partial(p, left > 0 ? (int)left : 0);
        }
      }
      v ^= flip;  // 0x80808080 turns unsigned bytes into signed ones minus 128
      reg[i] = v;
    }
  }

  __device__ static __forceinline__ void store(const v4i (&reg)[PER_THREAD], uint8_t *lds,
                                              int tid) {
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      int a, c;
      chunk_of(i, tid, a, c);
      *reinterpret_cast<v4i *>(lds + lds_offset(a, c)) = reg[i];
    }
  }

  // Fragment for one MFMA operand: lane l gets, for row (row0 + l%32), the 16
  // bytes k = 32*ks + 16*(l/32) .. +15 of the staged block.
  __device__ static __forceinline__ v4i fragment(const uint8_t *lds, int row0, int ks, int lane) {
    if (KC) {
      int r = row0 + (lane & 31);
      int c = ks * 2 + (lane >> 5);
      return *reinterpret_cast<const v4i *>(lds + lds_offset(r, c));
    } else {
      // ds_read_b64_tr_b8 (measured): inside each group of 16 lanes, lane 2t+h
      // supplies the address of 8 bytes: half h of a 16-byte row t; lane i
      // receives byte i of rows t = 0..7.  Rows are k, bytes are the index.
      int s = lane & 15;
      int col = row0 + ((lane >> 4) & 1) * 16 + (s & 1) * 8;
      int kbase = ks * 32 + (lane >> 5) * 16 + (s >> 1);
      v4i f;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        int q = kbase + t * 8;
        int off = q * R + (((col >> 4) ^ swz(q)) << 4) + (col & 15);
        v2i h = __builtin_amdgcn_ds_read_tr8_b64_v2i32(LDS_PTR(v2i, lds + off));
        f[2 * t] = h[0];
        f[2 * t + 1] = h[1];
      }
      return f;
    }
  }
};

}  // namespace mip
