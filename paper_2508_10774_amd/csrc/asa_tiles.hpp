// MFMA operand orderings, LDS swizzles and direct global->LDS tile copies shared by the
// forward and backward attention kernels (device code only).
#pragma once

#include "asa_common.hpp"

namespace asa {

// Row r of an MFMA A operand / accumulator splits as r = 8g + 4h + j (g<4, h<2, j<4); lane
// half h holds accumulator register 4g + j.
//
// kappa: which key of a 32-key group is loaded as A row r of S^T = K Q^T.  Chosen so that
// lane half h, registers 8t..8t+7 hold keys 16t + 8h + 0..7: exactly the 8 consecutive k
// slots that the B operand of the following 16-deep P^T step wants from that lane.
__device__ __forceinline__ int kappa(int r) {
  int g = r >> 3, h = (r >> 2) & 1, j = r & 3;
  return 16 * (g >> 1) + 8 * h + 4 * (g & 1) + j;
}
// rho: which channel of a 32-channel group is loaded as A row r of O^T = V^T P^T, chosen so
// that lane half h ends up with 16 consecutive channels 16h + (4g + j) of its query.
__device__ __forceinline__ int rho(int r) {
  int g = r >> 3, h = (r >> 2) & 1, j = r & 3;
  return 16 * h + 4 * g + j;
}

// LDS tiles are filled by direct global->LDS loads, which write 64 lanes x 16 B contiguously:
// rows cannot be padded, so 16-byte chunks are XOR-swizzled instead.  A K row holds D/8 chunks
// and is read by 16 lanes with 16 different rows (kappa) and one chunk index: chunk c of row r
// lives at position c ^ (r mod chunks).  A V^T row holds 8 chunks (128 B, half the banks) and is
// read through rho, whose 16 rows differ in row bits 0..2 and 4: position c ^ f(r) with f built
// from bits 1, 2, 4 separates the 8 rows of equal parity, parity itself picks the bank half.
template <int D>
__device__ __forceinline__ int k_swz(int row) {
  // D = 128: a row is all 64 banks, 16 rows need 16 positions; D = 64: a row is half the banks,
  // parity picks the half and the 8 rows of equal parity need 8 positions
  return D == 128 ? (row & 15) : ((row >> 1) & 7);
}
__device__ __forceinline__ int v_swz(int row) { return ((row >> 1) & 3) | (((row >> 4) & 1) << 2); }

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

// Swizzle of a row tile that is read both row-wise (16 lanes, 16 rows, one 16-byte chunk) and
// through the transposing LDS read (16 lanes: 4 consecutive rows x four 8-byte pieces).  With
// D = 128 the row's low two bits go to the chunk's high two bits, so that the 4 consecutive rows
// of a transposing read fall into 4 different quarters of the banks; any bijection of row mod 16
// serves the row-wise reads.  With D = 64 the k_swz pattern already serves both.
template <int D>
__device__ __forceinline__ int t_swz(int row) {
  return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((row >> 1) & 7);
}
// byte offset, in a t_swz row tile, of the 8-byte piece "row r, columns d4 .. d4 + 3" (d4 % 4 == 0)
template <int D>
__device__ __forceinline__ uint32_t tr_piece(int r, int d4) {
  return (uint32_t)((r * D + (((d4 >> 3) ^ t_swz<D>(r)) << 3) + (d4 & 4)) * 2);
}
// ds_read_b64_tr_b16: inside each group of 16 lanes, lane i receives as element j (j = 0..3) the
// 16-bit element i % 4 of the 8 bytes that lane 4 j + i / 4 of the group addressed.
__device__ __forceinline__ bf16x4 lds_read_tr16(const lds_char *p) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4 *)p);
#else
  return bf16x4{};
#endif
}

// One direct global->LDS load: every lane fetches 16 bytes from its own global address and the
// wavefront's 64 x 16 B land contiguously at the (wave-uniform) LDS address.  Counted by vmcnt.
// (The builtin only exists in the device pass; the host pass needs no body.)
__device__ __forceinline__ void lds_dma16(const void *src, void *lds_dst) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_global_load_lds(src, (lds_void *)lds_dst, 16, 0, 0);
#endif
}

// The same load with the address split into a wave-uniform 64-bit base (scalar registers) and
// a 32-bit per-lane byte offset: stepping to another tile then costs scalar adds only and the
// per-lane offsets stay 32 bits wide.  The compiler does not see this load: the caller waits
// with an explicit vmcnt before reading the LDS image, and a kernel that uses this form uses
// it for all of its direct loads (M0 is written here).
// lds_byte_addr is the wave-uniform LDS address (lds_addr_of() of the LDS array + offset).
// FORCE = false leaves the operands as the compiler has them (it must then know them to be
// uniform, or the assembler rejects the instruction).
template <bool FORCE = true>
__device__ __forceinline__ void lds_dma16_sv(const void *uniform_base, uint32_t lane_off,
                                             uint32_t lds_byte_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  if (!FORCE) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(lane_off), "s"(uniform_base), "s"(lds_byte_addr) : "memory");
    return;
  }
  // (readfirstlane costs nothing where the compiler already knows the value to be uniform and
  // puts it into scalar registers where it does not)
  const uint64_t b = reinterpret_cast<uint64_t>(uniform_base);
  // (the builtin returns a signed int: widen through uint32_t, or the low half sign-extends
  // into the high one)
  const uint64_t bu = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b) |
                      ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b >> 32)) << 32);
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(lane_off), "s"(bu), "s"((uint32_t)__builtin_amdgcn_readfirstlane(lds_byte_addr)) : "memory");
#endif
}
// The same (compiler-invisible) load with a full per-lane 64-bit address, and its 4-byte form.
__device__ __forceinline__ void lds_dma16_v(const void *lane_ptr, uint32_t lds_byte_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(lane_ptr), "s"((uint32_t)__builtin_amdgcn_readfirstlane(lds_byte_addr)) : "memory");
#endif
}
__device__ __forceinline__ void lds_dma4_v(const void *lane_ptr, uint32_t lds_byte_addr) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               :: "v"(lane_ptr), "s"((uint32_t)__builtin_amdgcn_readfirstlane(lds_byte_addr)) : "memory");
#endif
}
// LDS byte address of an object that the compiler knows to live in LDS (apply it to the
// __shared__ array itself, not to a pointer that travelled through generic address space)
#define ASA_LDS_ADDR_OF(shared_array) ((uint32_t)(uintptr_t)(::asa::lds_void *)(shared_array))

// ---------------------------------------------------------------------------------------
// Cooperative tile copies global -> LDS for a workgroup of WAVES wavefronts.  Per-lane byte
// offsets are computed once (init); every copy then costs only a wave-uniform base pointer.
// ---------------------------------------------------------------------------------------

// ROWS x D bf16 tile of a row-major [L][*] tensor (row pitch sL elements), rows past L - 1
// re-read row L - 1 (they are masked by the caller).  LDS image: unpadded rows, k_swz swizzle.
template <int ROWS, int D, int WAVES>
struct RowTileCopy {
  static constexpr int kChunks = D / 8;                       // 16-byte chunks per row
  static constexpr int kInstr = ROWS * kChunks / 64 / WAVES;  // wave instructions per copy
  uint32_t off[kInstr];
  int wave, lane;
  int64_t pitch_bytes;

  __device__ __forceinline__ void init(int wave_, int lane_, int64_t sL) {
    wave = wave_; lane = lane_; pitch_bytes = sL * 2;
#pragma unroll
    for (int i = 0; i < kInstr; ++i) {
      const int row = (wave * kInstr + i) * (64 / kChunks) + lane / kChunks;
      const int pos = lane % kChunks;
      off[i] = (uint32_t)(row * pitch_bytes + ((pos ^ k_swz<D>(row)) * 16));
    }
  }
  // copy the ROWS complete rows that start at byte address `base` into `stage`
  // row of the tile that instruction i of this lane copies; byte offset of its 1 KB LDS chunk
  __device__ __forceinline__ int row_of(int i) const {
    return (wave * kInstr + i) * (64 / kChunks) + lane / kChunks;
  }
  __device__ __forceinline__ uint32_t lds_chunk(int i) const { return (wave * kInstr + i) * 1024; }
  // (the *_at forms take the LDS byte address of the stage)
  __device__ __forceinline__ void issue_at(uint32_t stage, const char *base) const {
#pragma unroll
    for (int i = 0; i < kInstr; ++i) lds_dma16_sv(base, off[i], stage + (wave * kInstr + i) * 1024);
  }
  // instruction i of that copy alone (a kernel may spread the kInstr loads of a copy over time)
  __device__ __forceinline__ void issue_one_at(int i, uint32_t stage, const char *base) const {
    lds_dma16_sv(base, off[i], stage + (wave * kInstr + i) * 1024);
  }
  __device__ __forceinline__ void issue_one_at_ragged(int i, uint32_t stage, const char *base, int lim) const {
    if (lim < 0) {
      base += (int64_t)lim * pitch_bytes;
      lim = 0;
    }
    const int row = (wave * kInstr + i) * (64 / kChunks) + lane / kChunks;
    const uint32_t o = row > lim ? off[i] - (uint32_t)(row - lim) * (uint32_t)pitch_bytes : off[i];
    lds_dma16_sv(base, o, stage + (wave * kInstr + i) * 1024);
  }
  // the same for a tile whose rows past `lim` (relative to the tile) re-read row `lim`.
  // lim < 0 (the whole tile lies past the last row) moves the base back to that row first:
  // the per-lane offsets are unsigned and must not go negative.
  __device__ __forceinline__ void issue_at_ragged(uint32_t stage, const char *base, int lim) const {
    if (lim < 0) {
      base += (int64_t)lim * pitch_bytes;
      lim = 0;
    }
#pragma unroll
    for (int i = 0; i < kInstr; ++i) {
      const int row = (wave * kInstr + i) * (64 / kChunks) + lane / kChunks;
      const uint32_t o = row > lim ? off[i] - (uint32_t)(row - lim) * (uint32_t)pitch_bytes : off[i];
      lds_dma16_sv(base, o, stage + (wave * kInstr + i) * 1024);
    }
  }
  // copy rows [row0, row0 + ROWS) of `tensor` (slab base) into `stage`
  __device__ __forceinline__ void issue(bf16 *stage, const bf16 *tensor, int row0, int L) const {
    const char *base = reinterpret_cast<const char *>(tensor) + (int64_t)row0 * pitch_bytes;
    const int lim = L - 1 - row0;   // last valid row of the tile
    if (lim >= ROWS - 1) {
#pragma unroll
      for (int i = 0; i < kInstr; ++i) lds_dma16(base + off[i], stage + (wave * kInstr + i) * 512);
    } else {
#pragma unroll
      for (int i = 0; i < kInstr; ++i) {
        const int row = (wave * kInstr + i) * (64 / kChunks) + lane / kChunks;
        const char *src = base + off[i];
        if (row > lim) src -= (int64_t)(row - lim) * pitch_bytes;
        lds_dma16(src, stage + (wave * kInstr + i) * 512);
      }
    }
  }
};

// D x 64 slice (columns [col0, col0 + 64)) of a transposed tile stored as [D][BLK] bf16.
// LDS image: [D][64], v_swz swizzle.
template <int BLK, int D, int WAVES>
struct ColTileCopy {
  static constexpr int kInstr = D * 8 / 64 / WAVES;
  uint32_t off[kInstr];
  int wave;

  __device__ __forceinline__ void init(int wave_, int lane) {
    wave = wave_;
#pragma unroll
    for (int i = 0; i < kInstr; ++i) {
      const int row = (wave * kInstr + i) * 8 + lane / 8;
      off[i] = (uint32_t)((row * BLK + (((lane % 8) ^ v_swz(row)) * 8)) * 2);
    }
  }
  __device__ __forceinline__ void issue(bf16 *stage, const bf16 *tile, int col0) const {
    const char *base = reinterpret_cast<const char *>(tile + col0);
#pragma unroll
    for (int i = 0; i < kInstr; ++i) lds_dma16(base + off[i], stage + (wave * kInstr + i) * 512);
  }
  __device__ __forceinline__ void issue_at(uint32_t stage, const char *base) const {
#pragma unroll
    for (int i = 0; i < kInstr; ++i) lds_dma16_sv(base, off[i], stage + (wave * kInstr + i) * 1024);
  }
  template <bool FORCE = true>
  __device__ __forceinline__ void issue_one_at(int i, uint32_t stage, const char *base) const {
    lds_dma16_sv<FORCE>(base, off[i], stage + (wave * kInstr + i) * 1024);
  }
};

// The same two copies (the row tile with the t_swz swizzle) for a kernel that cannot spare registers for the offset tables: nothing
// is kept per lane, each offset is rebuilt from the lane number where it is used (a few integer
// instructions per load).  The caller passes the lane number through an empty asm statement
// inside its loop, so that the compiler does not hoist the offsets back into registers.
template <int ROWS, int D, int WAVES>
struct LeanRowTileCopy {
  static constexpr int kChunks = D / 8;                       // 16-byte chunks per row
  static constexpr int kRowsPer = 64 / kChunks;               // rows per wave instruction
  static constexpr int kInstr = ROWS * kChunks / 64 / WAVES;  // wave instructions per copy
  static_assert((kInstr * kRowsPer) % 16 == 0, "a wave's first row must be a multiple of 16");

  // copy rows [row0, row0 + ROWS) of `tensor` (slab base, row pitch sL elements) to the LDS
  // byte address `stage`; rows past L - 1 re-read row L - 1.  The loads are of the kind the
  // compiler does not see: the caller waits with an explicit vmcnt before reading the tile.
  static __device__ __forceinline__ void issue(uint32_t stage, const bf16 *tensor, int row0, int L,
                                               int64_t sL, int wave, int lane) {
    const int64_t pitch = sL * 2;
    const int lane_row = lane / kChunks, pos = lane % kChunks;
    const char *base = reinterpret_cast<const char *>(tensor) + (int64_t)row0 * pitch;
    const int lim = L - 1 - row0;   // last valid row of the tile
    if (lim >= ROWS - 1) {
      const uint32_t lane_row_off = (uint32_t)lane_row * (uint32_t)pitch;
#pragma unroll
      for (int i = 0; i < kInstr; ++i) {
        const int r0 = (wave * kInstr + i) * kRowsPer;                    // wave-uniform
        const int sw = t_swz<D>(((i * kRowsPer) & 15) + lane_row);        // = t_swz(r0 + lane_row)
        const uint32_t lo = lane_row_off + (uint32_t)((pos ^ sw) * 16);
        lds_dma16_sv(base + (int64_t)r0 * pitch, lo, stage + (wave * kInstr + i) * 1024);
      }
    } else {
#pragma unroll
      for (int i = 0; i < kInstr; ++i) {
        const int row = (wave * kInstr + i) * kRowsPer + lane_row;
        const int sw = t_swz<D>(row);
        const int src_row = row > lim ? lim : row;                        // may be negative
        lds_dma16_v(base + (int64_t)src_row * pitch + (pos ^ sw) * 16, stage + (wave * kInstr + i) * 1024);
      }
    }
  }
};

// LDS address (elements) of the A fragment "row r, 16-byte chunk c" in the two images
template <int D>
__device__ __forceinline__ int row_tile_elem(int r, int c) { return r * D + ((c ^ k_swz<D>(r)) * 8); }
__device__ __forceinline__ int col_tile_elem(int r, int c) { return r * 64 + ((c ^ v_swz(r)) * 8); }

}  // namespace asa
