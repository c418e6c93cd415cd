// LDS tile layouts and global->LDS movers shared by the GEMM and attention kernels.
//
// An operand tile is R rows (the non-contracted index: m, n, query or key position) by 64
// contraction elements, held as 16-byte chunks of 8 consecutive contraction elements, so that an
// MFMA fragment (row = lane%32, 8 contraction values) is one ds_read_b128.
//
// Two layouts, chosen by how the operand lies in HBM:
//   KC ("contraction contiguous", memory [row][k]): chunks are copied as they are.  Slot function
//      lds_slot_kc() puts a pair of rows on one 256-byte line and XOR-swizzles the chunk index, so
//      that both the copy (8 chunks x 2 rows per 16 lanes) and the fragment read (16 rows, one
//      chunk) touch 16 distinct 16-byte bank groups.
//   KS ("contraction strided", memory [k][row]): a thread gathers an 8(k) x 4(row) block with eight
//      8-byte loads, transposes it in registers with v_perm_b32 and writes four chunks.  Slot function
//      lds_slot_ks() is chunk-major inside 16-row groups with a rotation, so that the writes
//      (rows 4 apart) and the fragment reads (consecutive rows) are both conflict-free.
#pragma once
#include "common.h"

constexpr int TILE_K = 64;             // contraction elements per LDS tile
constexpr int TILE_ROW_BYTES = 128;    // 64 bf16

DEV int lds_slot_kc(int r, int kc) {
  return ((r >> 1) << 4) + ((((r ^ (r >> 3)) & 1) << 3) | (kc ^ ((r >> 1) & 7)));
}
DEV int lds_slot_ks(int r, int kc) {
  return ((r >> 4) << 7) + (kc << 4) + (((r & 15) + ((r >> 4) & 3)) & 15);
}
template <bool KS>
DEV int lds_slot(int r, int kc) { return KS ? lds_slot_ks(r, kc) : lds_slot_kc(r, kc); }

template <bool KS>
DEV bf16x8 lds_read_frag(const uint8_t* tile, int r, int kc) {
  return *reinterpret_cast<const bf16x8*>(tile + (lds_slot<KS>(r, kc) << 4));
}

// ---- buffer resources -------------------------------------------------------------------------
// Global reads go through raw buffer loads: an offset at or beyond num_records returns zeros, which
// clips ragged tiles without branches.  Out-of-tile lanes are given the offset BUF_OOB.
typedef __amdgpu_buffer_rsrc_t buf_rsrc;
constexpr uint32_t BUF_OOB = 0x80000000u;      // operands are validated to be smaller than 2 GiB
DEV buf_rsrc make_rsrc(const void* base, long bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// ---- KC mover: memory [row][k], row stride ld elements ------------------------------------------
template <int R, int NT>
struct MoverKC {
  static_assert((R * 8) % NT == 0 && NT % 8 == 0, "tile chunks must divide over the threads");
  static constexpr int CH = R * 8 / NT;
  u32x4 regs[CH];
  uint32_t base[CH];   // byte offset of this thread's chunk at k = 0, or BUF_OOB for clipped rows
  int kofs;            // contraction offset of this thread's chunks inside a tile

  // rows [row0, row0+R) of the operand, clipped to row_end
  DEV void init(int ld, int row0, int row_end, int tid) {
    kofs = (tid & 7) * 8;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      int gr = row0 + ((tid + i * NT) >> 3);
      base[i] = gr < row_end ? (uint32_t)(gr * ld + kofs) * 2u : BUF_OOB;
    }
  }
  // contraction range [k0, k0+64) clipped to k_end (chunk granular: k_end % 8 == 0)
  DEV void load(buf_rsrc rs, int k0, int k_end, uint32_t row_byte_off = 0) {
    const bool ok = k0 + kofs < k_end;
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      uint32_t off = ok ? base[i] + (uint32_t)k0 * 2u + row_byte_off : BUF_OOB;
      regs[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
    }
  }
  DEV void store(uint8_t* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      int c = tid + i * NT;
      *reinterpret_cast<u32x4*>(tile + (lds_slot_kc(c >> 3, c & 7) << 4)) = regs[i];
    }
  }
};

// ---- KS mover: memory [k][row], k stride ld elements ---------------------------------------------
// ColMap maps a tile-local row index (multiple of 4) to the element offset inside a memory row, or
// a negative value if that group of 4 lies outside the operand.  Contraction indices at or beyond
// the operand's last memory row fall outside the buffer extent and read as zero by themselves.
struct IdentityCols {
  int row0, row_end;
  DEV int operator()(int r) const { int g = row0 + r; return g < row_end ? g : -1; }
};

// PERM: chunk kb of a 64-wide contraction tile gathers the contraction indices
//   16 (kb/2) + 4 (kb%2) + {0,1,2,3, 8,9,10,11}
// instead of 8 kb + {0..7}.  That is the order in which a lane of a 32x32 MFMA accumulator holds
// its 16 rows, so an accumulator converted to bf16 can be fed back as the other operand of the
// next product without leaving registers (attention: P -> P V, dS -> dS K, ...).
template <int R, int NT, bool PERM = false>
struct MoverKS {
  static constexpr int NBLK = R * 2;                       // 8x4 blocks in the tile
  static constexpr int NB = (NBLK + NT - 1) / NT;          // blocks per thread (last may be idle)
  static_assert(R % 16 == 0, "rows come in groups of 16");
  u32x2 regs[NB][8];
  uint32_t base[NB];
  int ld2;                                // bytes per memory row

  template <class ColMap>
  DEV void init(int ld, const ColMap& cols, int tid) {
    ld2 = ld * 2;
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      int id = tid + i * NT;
      int ib4 = id % (R / 4), kb = id / (R / 4);
      int gc = (NBLK % NT == 0 || id < NBLK) ? cols(ib4 * 4) : -1;
      int kstart = PERM ? (kb >> 1) * 16 + (kb & 1) * 4 : kb * 8;
      base[i] = gc >= 0 ? (uint32_t)(kstart * ld + gc) * 2u : BUF_OOB;
    }
  }
  DEV void load(buf_rsrc rs, int k0, int /*k_end*/) {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const int rofs = PERM ? (r & 3) + (r >> 2) * 8 : r;
        uint32_t off = base[i] + (uint32_t)((k0 + rofs) * ld2);
        regs[i][r] = __builtin_amdgcn_raw_buffer_load_b64(rs, off, 0, 0);
      }
    }
  }
  DEV void store(uint8_t* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      int id = tid + i * NT;
      if (NBLK % NT != 0 && id >= NBLK) continue;
      int ib4 = id % (R / 4), kb = id / (R / 4);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
        u32x4 o;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
          o[kk] = __builtin_amdgcn_perm(regs[i][2 * kk + 1][c >> 1], regs[i][2 * kk][c >> 1], sel);
        *reinterpret_cast<u32x4*>(tile + (lds_slot_ks(ib4 * 4 + c, kb) << 4)) = o;
      }
    }
  }
};
