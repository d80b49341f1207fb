// Direct-to-LDS staging, per-lane fragment offsets and the block-id decoding.
#ifndef VARLEN_ATTN_STAGING_HPP_
#define VARLEN_ATTN_STAGING_HPP_

#include "tiles.hpp"

namespace {

// ----------------------------------------------------------------------------------------
// Global -> LDS staging without registers (global_load_lds_dwordx4): the 64 lanes of a wave
// write 1 KiB contiguous in LDS starting at the wave-uniform address in M0, each lane taking
// its 16 bytes from its own global address.  A stage holds kSub = 32 rows of a [rows][D] tile;
// the XOR swizzle is applied on the global side (lane of physical chunk pc in row r fetches
// logical chunk pc ^ swz(r)).  Rows past `row_last` are clamped to it: they are finite
// duplicates that the causal mask (or a zero P) removes, never garbage.
//
// The loads are invisible to the compiler's wait-count bookkeeping (inline asm), which is
// the point: a compiler-inserted wait would be vmcnt(0) before every LDS read.  The kernels
// wait explicitly with wait_vm<N>() and publish with a barrier.  Extra outstanding loads can
// only make compiler-inserted vmcnt waits longer, never too short (in-order completion).
// ----------------------------------------------------------------------------------------
constexpr int kSub = 32;  // rows per pipeline stage

// base: wave-uniform 64-bit address; voff: this lane's unsigned byte offset from it
__device__ __forceinline__ void dma16(unsigned long long base, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(base), "s"(lds_addr)
               : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt immediate");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// vmcnt(0) as an instruction the compiler's wait-count pass can see (expcnt, lgkmcnt untouched)
__device__ __forceinline__ void wait_all_vm_visible() { __builtin_amdgcn_s_waitcnt(0x0F70); }
__device__ __forceinline__ unsigned lds_addr_of(const void* p) {
  return (unsigned)(size_t)(const __attribute__((address_space(3))) char*)p;
}
__device__ __forceinline__ unsigned long long uniform64(const void* p) {
  const unsigned long long v = (unsigned long long)(size_t)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return ((unsigned long long)hi << 32) | lo;
}

// Loads 32-row stages of a [rows][D] bf16 tile whose rows are `stride_bytes` apart.  The
// per-lane part of the address is a 32-bit offset fixed at init; the stage's first row goes
// into the wave-uniform base, so a stage costs no vector arithmetic unless it runs past
// `row_last` (then rows are clamped lane by lane).
template <int D, int ROWS = kSub>
struct StageLoader {
  static constexpr int kRowsPerInstr = 1024 / (D * 2);      // 4 (D=128), 8 (D=64)
  static constexpr int kInstr = ROWS / kRowsPerInstr;       // wave-level loads per stage
  static constexpr int kPerWave = kInstr / 4;               // 4 waves share a stage
  int row_in_stage[kPerWave];
  unsigned col_bytes[kPerWave];
  unsigned voff[kPerWave];
  unsigned stride_bytes;
  __device__ __forceinline__ void init(int wave, int lane, unsigned stride_bytes_) {
    stride_bytes = stride_bytes_;
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const int j = wave + 4 * i;
      const int r = kRowsPerInstr * j + lane / (D / 8), pc = lane % (D / 8);
      row_in_stage[i] = r;
      col_bytes[i] = (unsigned)((pc ^ swz<D>(r)) * 16);
      voff[i] = (unsigned)r * stride_bytes + col_bytes[i];
    }
  }
  // tile rows [row0, row0 + ROWS) of `base` -> LDS at `lds`; rows above row_last are clamped
  __device__ __forceinline__ void issue(const __bf16* base, int row0, int row_last, unsigned lds,
                                        int wave) const {
    issue_at(uniform64(reinterpret_cast<const char*>(base) + (size_t)row0 * stride_bytes), row0,
             row_last, lds, wave);
  }
  // the same with the wave-uniform address of row `row0` already at hand (a chain keeps it in
  // scalar registers and moves it on by one stage per call)
  __device__ __forceinline__ void issue_at(unsigned long long b, int row0, int row_last,
                                           unsigned lds, int wave) const {
    if (row0 + ROWS - 1 <= row_last) {
#pragma unroll
      for (int i = 0; i < kPerWave; ++i)
        dma16(b, voff[i], __builtin_amdgcn_readfirstlane(lds + (wave + 4 * i) * 1024));
    } else {
#pragma unroll
      for (int i = 0; i < kPerWave; ++i) {
        const int r = min(row_in_stage[i], row_last - row0);   // row_last >= row0 always
        dma16(b, (unsigned)r * stride_bytes + col_bytes[i],
              __builtin_amdgcn_readfirstlane(lds + (wave + 4 * i) * 1024));
      }
    }
  }
};

// 64 consecutive floats (clamped at index `last`) -> 256 bytes of LDS, one wave-level load
__device__ __forceinline__ void dma_floats64(const float* base, int first, int last, unsigned lds,
                                             int lane) {
  const unsigned long long b = uniform64(base + first);
  unsigned voff = (unsigned)lane * 4;
  if (first + 63 > last) voff = (unsigned)min(lane, last - first) * 4;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :
               : "v"(voff), "s"(b), "s"(__builtin_amdgcn_readfirstlane(lds))
               : "memory");
}

// per-lane byte offsets (inside a stage) of the two kinds of fragment reads
template <int D>
struct FragOffsets {
  int row_frag[D / 16];     // A/B row fragment of row c, k slice kk: chunk 2kk + h
  int trans[D / 32][2];     // transposed fragment, column block db, rows 4h + i/4 (+8)
  __device__ __forceinline__ void init(int lane) {
    const int h = lane >> 5, c = lane & 31, i = lane & 15, b16 = (lane >> 4) & 1;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) row_frag[kk] = chunk_off<D>(c, 2 * kk + h);
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int second = 0; second < 2; ++second) {
        const int row = 4 * h + (i >> 2) + 8 * second;
        const int chunk = 4 * db + 2 * b16 + ((i & 3) >> 1);
        trans[db][second] = chunk_off<D>(row, chunk) + (i & 1) * 8;
      }
  }
};
// transposed A operand for rows 16 cc + {4h.., 8 + 4h..} of a stage, column block db
template <int D>
__device__ __forceinline__ bf16x8 read_trans(const char* stage, const FragOffsets<D>& fo, int cc,
                                             int db) {
  bf16x4 lo = lds_read_tr(stage + fo.trans[db][0] + cc * 16 * D * 2);
  bf16x4 hi = lds_read_tr(stage + fo.trans[db][1] + cc * 16 * D * 2);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// the same from two explicit addresses (rows .. and rows + 8 ..)
__device__ __forceinline__ bf16x8 lds_read_tr8(const char* lo_addr, const char* hi_addr) {
  bf16x4 lo = lds_read_tr(lo_addr);
  bf16x4 hi = lds_read_tr(hi_addr);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).  Decode the id so
// that all units of one head land on the same XCDs and share its K/V (or Q/dO) lines in L2;
// where a head has several XCDs, runs of kUnitRun consecutive units stay on one of them: the
// chunks of one tile are neighbours in the unit list and read the same Q (dO, O; K, V) rows.
constexpr int kUnitRun = 4;
__device__ __forceinline__ void decode_block(int bid, int Hq, int& unit, int& head) {
  constexpr int kXcds = 8;
  const int xcd = bid % kXcds, local = bid / kXcds;
  if (kXcds % Hq == 0) {
    const int per = kXcds / Hq;          // XCDs per head
    head = xcd % Hq;
    unit = (local / kUnitRun) * (kUnitRun * per) + (xcd / Hq) * kUnitRun + local % kUnitRun;
  } else if (Hq % kXcds == 0) {
    const int per = Hq / kXcds;          // heads per XCD
    head = xcd + kXcds * (local % per);
    unit = local / per;
  } else {
    unit = bid / Hq;
    head = bid % Hq;
  }
}
// grid that covers `units` units of every head under decode_block (whole runs on every XCD)
inline unsigned grid_for(int units, int Hq) {
  const long long round = 8 * kUnitRun;
  return (unsigned)(((long long)units * Hq + round - 1) / round * round);
}

}  // namespace

#endif  // VARLEN_ATTN_STAGING_HPP_
