// Device-side building blocks shared by the gfx950 kernels of the hybrid
// attention library: vector types, the bf16 MFMA wrapper with its operand
// layout, LDS tile staging and the chunk bookkeeping formulas.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rehyat {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short i16x4;

typedef uint16_t bf16_t;  // storage type of a bf16 value

constexpr int kWave = 64;

// ---------------------------------------------------------------------------
// Chunk bookkeeping (section 3.2 token layout; Eq. 12; Eq. 13).  The host
// entry point rehyat_chunk_plan and every kernel use this one function.
// ---------------------------------------------------------------------------
struct ChunkRange {
  int64_t q_lo, q_hi;  // query tokens of the chunk
  int64_t s_lo, s_hi;  // softmax window
  int64_t l_hi;        // causal linear set is [0, l_hi)
};

__host__ __device__ inline int num_chunks(int T, int chunk) {
  // 64-bit: chunk may be as large as INT_MAX ("one chunk covers everything")
  return (int)(((int64_t)T + chunk - 1) / chunk);
}

__host__ __device__ inline ChunkRange chunk_range(int T, int HW, int chunk, int overlap, int t) {
  ChunkRange r;
  int64_t f0 = (int64_t)t * chunk;
  int64_t f1 = f0 + chunk;
  if (f1 > T) f1 = T;
  r.q_lo = f0 * HW;
  r.q_hi = f1 * HW;
  int64_t s = r.q_lo - (int64_t)overlap * HW;
  r.s_lo = s < 0 ? 0 : s;
  r.s_hi = r.q_hi;
  r.l_hi = r.s_lo;
  return r;
}

// ---------------------------------------------------------------------------
// v_mfma_f32_32x32x16_bf16: D[32x32] += A[32x16] * B[16x32].
// Lane l = 32*g + r holds A[r][8g .. 8g+7] and B[8g .. 8g+7][r]; accumulator
// register 4*i + j of lane l holds D[8i + 4g + j][r].
// Because the contraction index may be permuted freely as long as A and B
// agree, an accumulator (rows 8i+4g+j in registers) converts in place into
// the B operand of a following product: registers 8s .. 8s+7 become the eight
// k-values of k-step s, which are rows 16s + {4g..4g+3, 8+4g..8+4g+3}.  The
// matching A operand is read from a tile whose 16-element groups are stored
// with their two middle quads swapped ("quad-swapped" layout, see
// stage_tile<true>), or through transposing LDS reads for row-major data.
// ---------------------------------------------------------------------------
__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ float bf16_round(float x) {
  // value of x after round-to-nearest-even to bf16
  uint32_t u = pack_bf16(x, 0.f) << 16;
  return __builtin_bit_cast(float, u);
}

// Registers 8s .. 8s+7 of an accumulator -> one bf16 B operand.
__device__ __forceinline__ bf16x8 acc_to_operand(const f32x16& c, int s) {
  u32x4 p;
  p[0] = pack_bf16(c[8 * s + 0], c[8 * s + 1]);
  p[1] = pack_bf16(c[8 * s + 2], c[8 * s + 3]);
  p[2] = pack_bf16(c[8 * s + 4], c[8 * s + 5]);
  p[3] = pack_bf16(c[8 * s + 6], c[8 * s + 7]);
  return __builtin_bit_cast(bf16x8, p);
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes,
// lane i passes the address of 4 consecutive bf16 of row (i / 4) at column
// group (i % 4) of a 4 x 16 block and receives column i of that block, rows
// 0..3.
__device__ __forceinline__ i16x4 lds_read_tr(const bf16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (__attribute__((address_space(3))) i16x4*)(p));
}

// ---------------------------------------------------------------------------
// LDS tiles are [rows][ROWBYTES] with unpadded rows, filled by direct
// global->LDS loads (each wave instruction moves 1 KB to consecutive LDS
// bytes, so rows cannot be padded).  Bank conflicts are avoided by permuting
// the 16-byte chunks of a row: chunk c of row `row` is stored at chunk position
// c ^ swz(row).  swz is a bijection of the rows that a 32x32x16 A-fragment read
// touches together (16 consecutive rows, same chunk) onto chunk positions, and
// it also separates the 4 consecutive rows that one transposing read touches.
// ---------------------------------------------------------------------------
template <int ROWBYTES>
__device__ __forceinline__ int swz(int row) {
  // 256- and 512-byte rows: 16 consecutive rows land on 16 distinct chunk positions (the
  // permutation touches the low four bits of the chunk index only)
  if (ROWBYTES == 256 || ROWBYTES == 512) return ((row & 3) << 2) | ((row >> 2) & 3);
  return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);                  // 128-byte rows, 8 chunks
}

// byte offset of element (row, col) inside a tile whose rows hold ROWBYTES/2 bf16
template <int ROWBYTES>
__device__ __forceinline__ int tile_off(int row, int col) {
  return row * ROWBYTES + ((((col >> 3) ^ swz<ROWBYTES>(row)) << 4) | ((col & 7) << 1));
}

// Direct loads of one tile.  Wave w of NW moves the 1 KB blocks w, w+NW, ...; lane i of
// a block fills LDS chunk slot i, so it fetches the global chunk that the
// swizzle assigns to that slot.  `rowaddr(R)` gives the byte offset, from
// `gbase`, of the global row segment that becomes tile row R.
template <int ROWBYTES, int TILE_BYTES, int NW, typename RowAddr>
__device__ __forceinline__ void tile_load_direct(const char* gbase, char* lds_tile, int wave, int lane,
                                                 RowAddr rowaddr) {
  constexpr int CPR = ROWBYTES / 16;     // chunks per row
  constexpr int RPB = 1024 / ROWBYTES;   // rows per 1 KB block
  constexpr int NBLK = TILE_BYTES / 1024;
  static_assert(NBLK % NW == 0, "blocks of a tile are dealt evenly to the waves");
#pragma unroll
  for (int n = 0; n < NBLK / NW; ++n) {
    const int blk = wave + NW * n;
    const int R = blk * RPB + lane / CPR;
    const int c = (lane % CPR) ^ swz<ROWBYTES>(R);
    const char* src = gbase + (uint32_t)(rowaddr(R) + c * 16);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                     (__attribute__((address_space(3))) void*)(lds_tile + blk * 1024), 16, 0, 0);
  }
}

// Raw buffer descriptor for direct loads.  The hardware's range check covers only
// the per-lane offset (never the scalar offset), so the descriptor is left open
// ended and callers keep every access inside their tensors themselves.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}

// Same tile fill as tile_load_direct for row maps that split into a block part and a
// row-in-block part, rowaddr(blk * RPB + j) == rowaddr(blk * RPB) + rowaddr(j) for j < RPB
// (RPB = rows per 1 KB block): the per-lane offset is then the same for every block a
// wave moves, and the block part, the tile offset `soff` (bytes from the descriptor's
// base) and the LDS address are all wave-uniform, so a load costs no vector ALU work.
// `wave` must be wave-uniform in the compiler's eyes (readfirstlane).
template <int ROWBYTES, int TILE_BYTES, int NW, typename RowAddr>
__device__ __forceinline__ void tile_load_buffer(__amdgpu_buffer_rsrc_t rsrc, int soff, char* lds_tile,
                                                 int wave, int lane, RowAddr rowaddr) {
  constexpr int CPR = ROWBYTES / 16;
  constexpr int RPB = 1024 / ROWBYTES;
  constexpr int NBLK = TILE_BYTES / 1024;
  static_assert(NBLK % NW == 0, "blocks of a tile are dealt evenly to the waves");
  const int j = lane / CPR;
#pragma unroll
  for (int n = 0; n < NBLK / NW; ++n) {
    const int blk = wave + NW * n;
    // the chunk swizzle looks at the low bits of the block index only: with NW a multiple
    // of 4 every block of a wave shares one per-lane offset, otherwise two alternate
    const int c = (lane % CPR) ^ swz<ROWBYTES>((NW % 4 == 0 ? wave : blk) * RPB + j);
    const int voff = rowaddr(j) + c * 16;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(lds_tile + blk * 1024),
                                             16, voff, soff + rowaddr(blk * RPB), 0, 0);
  }
}

// The same direct load written as inline asm, for kernels that rotate tile buffers at run
// time.  The compiler orders every LDS read after any direct load it can see that might
// write the same object, by waiting for ALL outstanding loads -- right for one buffer,
// but with buffers picked by a run-time index it cannot tell the tile being read from the
// tile being prefetched, and the wait would undo the prefetch.  Loads issued here are
// invisible to that analysis; callers order them against the reads themselves with
// wait_loads_and_barrier.  `rsrc` is the descriptor as four scalar words, `soff` a
// wave-uniform byte offset, `lds_addr` the wave-uniform LDS byte address of the 1 KB block
// (lane i writes bytes [16 i, 16 i + 16) of it).
__device__ __forceinline__ u32x4 make_rsrc_words(const void* base) {
  const uint64_t b = (uint64_t)base;
  u32x4 w;
  w[0] = __builtin_amdgcn_readfirstlane((uint32_t)b);
  w[1] = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32) & 0xffffu);
  w[2] = 0x7fffffffu;   // open ended, as in make_rsrc
  w[3] = 0x00020000u;
  return w;
}
__device__ __forceinline__ void direct_load_16(u32x4 rsrc, int voff, int soff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               ::"s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}
// Four bytes per lane: lane i writes bytes [4 i, 4 i + 4) of the 256-byte block at lds_addr.
__device__ __forceinline__ void direct_load_4(u32x4 rsrc, int voff, int soff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
               ::"s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

// One tile through direct_load_16.  Rows at or beyond `valid` re-read the last valid row
// (finite values; callers mask what they compute from them).  Wave w of NW moves the 1 KB
// blocks w, w+NW, ...; `soff` is the tile's byte offset from the descriptor's base.
template <int ROWBYTES, int TILE_BYTES, int NW>
__device__ __forceinline__ void tile_load_asm(u32x4 rsrc, int soff, uint32_t lds_tile, int wave, int lane,
                                              int valid) {
  constexpr int CPR = ROWBYTES / 16;     // chunks per row
  constexpr int RPB = 1024 / ROWBYTES;   // rows per 1 KB block
  constexpr int NBLK = TILE_BYTES / 1024;
  static_assert(NBLK % NW == 0, "blocks of a tile are dealt evenly to the waves");
#pragma unroll
  for (int n = 0; n < NBLK / NW; ++n) {
    const int blk = wave + NW * n;
    int R = blk * RPB + lane / CPR;
    const int c = (lane % CPR) ^ swz<ROWBYTES>(R);
    if (R >= valid) R = valid - 1;
    direct_load_16(rsrc, R * ROWBYTES + c * 16, soff, lds_tile + blk * 1024);
  }
}

// tile_load_asm with one per-lane offset for every block a wave moves when the tile is full
// (valid == 64): block b of a wave differs from its first block by whole multiples of 16
// rows, which the chunk permutation does not see, so the block part goes into the scalar
// offset and the per-lane offset is loop-invariant (one register per tile shape instead of
// one per load).  `voff_full` is that offset, from tile_voff_full; a ragged tile takes the
// general path.
template <int ROWBYTES, int NW>
__device__ __forceinline__ int tile_voff_full(int wave, int lane) {
  constexpr int CPR = ROWBYTES / 16;
  constexpr int RPB = 1024 / ROWBYTES;
  static_assert((NW * RPB) % 16 == 0, "blocks of a wave are whole multiples of 16 rows apart");
  const int j = lane / CPR;
  return j * ROWBYTES + (((lane % CPR) ^ swz<ROWBYTES>(wave * RPB + j)) << 4);
}
template <int ROWBYTES, int TILE_BYTES, int NW>
__device__ __forceinline__ void tile_load_fast(u32x4 rsrc, int soff, uint32_t lds_tile, int wave, int lane,
                                               int valid, int voff_full) {
  constexpr int NBLK = TILE_BYTES / 1024;
  static_assert(NBLK % NW == 0, "blocks of a tile are dealt evenly to the waves");
  if (valid >= 64) {
#pragma unroll
    for (int n = 0; n < NBLK / NW; ++n) {
      const int blk = wave + NW * n;
      direct_load_16(rsrc, voff_full, soff + blk * 1024, lds_tile + blk * 1024);
    }
  } else {
    // at most once per token range: keep its per-load offsets from being computed ahead of
    // the loop and held in registers (the empty asm hides that they are loop-invariant)
    asm volatile("" : "+s"(valid), "+v"(lane));
    tile_load_asm<ROWBYTES, TILE_BYTES, NW>(rsrc, soff, lds_tile, wave, lane, valid);
  }
}

// Wait until at most N of this wave's direct loads are outstanding (and all of
// its LDS accesses are done), then workgroup barrier.  Written as one asm block:
// the compiler's own barrier would wait for every outstanding direct load and
// so serialise the prefetch with the computation.
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}
// Wait for this wave's LDS accesses only, then workgroup barrier (outstanding global
// stores and loads stay in flight).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ __forceinline__ bf16x8 join_tr(i16x4 lo, i16x4 hi) {
  typedef __attribute__((__vector_size__(8 * sizeof(short)))) short i16x8;
  i16x8 v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, v);
}

// Combine a per-lane value across the two 32-lane halves of the wave with
// v_permlane32_swap: it exchanges the high half of its first register with the
// low half of its second, so starting from two copies of x one register ends
// up holding the low half's values in all lanes and the other the high half's.
// Written as inline asm with both registers read-write (the compiler builtin
// loses track of the second result when both inputs are copies of one value);
// the leading s_nop covers the VALU-write -> permlane-read hazard.
__device__ __forceinline__ void half_swap(float& a, float& b) {
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float half_swap_max(float x) {
  float a = x, b = x;
  half_swap(a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float half_swap_sum(float x) {
  float a = x, b = x;
  half_swap(a, b);
  return a + b;
}

// Workgroup index -> logical work item so that consecutive logical items run
// on the same XCD: hardware deals workgroups round-robin over the 8 XCDs, each
// with its own L2, and items that share K/V or weights are consecutive.
__device__ __forceinline__ int xcd_swizzle(int wg, int per_xcd) {
  return (wg & 7) * per_xcd + (wg >> 3);
}

}  // namespace rehyat
