// Building blocks shared by the stripe kernels of the low-rank blocks on the MFMA path (k_proj_mfma.hip,
// k_proj_keep.hip): tile geometry, range-checked buffer access, the two bf16 (hi, lo) images of a factor,
// opaque LDS fragment reads with explicit waits, the role barrier and the direct global -> LDS copy.
#pragma once
#include "adapm_plan.h"
#include "ew_math.h"

namespace adapm {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int BM = 128;    // rows per stripe (one workgroup)
constexpr int BK = 64;     // columns per chunk (both passes)
constexpr int GS = BK + 8; // LDS row stride of the G tile (elements): 16-byte fragment reads hit all banks
constexpr int CS = BK + 8; // LDS row stride of the fp32 C tile
constexpr int NT = 1024;   // threads: waves 0-7 feed the matrix cores, waves 8-15 stream G, W and do the element-wise work

// Range-checked buffer access: a lane whose offset is at or beyond the descriptor's size reads zeros /
// writes nothing, so ragged edges need no branches and the compiler can count outstanding loads.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr unsigned OOB = 0x80000000u;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buf_load16(__amdgpu_buffer_rsrc_t r, unsigned off) {
  const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void buf_store16(__amdgpu_buffer_rsrc_t r, unsigned off, uint4 q) {
  u32x4 v;
  v.x = q.x; v.y = q.y; v.z = q.z; v.w = q.w;
  __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)off, 0, 0);
}

// Geometry of the two images of Q (per 64-column chunk, bf16 (hi, lo)):
//  * pass 1, fragment-major: [k-step][r-tile][hi|lo][lane][8]; lane l holds Q[32 tile + l%32][64 c + 16 kk + 8 (l/32) .. +7]
//  * pass 2, rows of Q^T:    [hi|lo][column j][R], the 16-byte pieces of a row XOR-swizzled with the row
//    index so that the fragment reads of 16 consecutive rows fall on different banks without padding.
__host__ __device__ constexpr int qf_chunk_bytes(int R) { return (BK / 16) * (R / 32) * 2 * 64 * 16; }
__host__ __device__ constexpr int timg_chunk_bytes(int R) { return 2 * BK * R * 2; }
__host__ __device__ __forceinline__ int timg_piece(int R, int j, int q) {   // physical 16-byte piece of logical piece q of row j
  const int pr = R / 8, rp = 16 / pr;
  return q ^ ((j / rp) & (pr - 1));
}

// LDS access of the matrix-core waves inside the role loops.  The compiler cannot see that a fragment
// read never touches the buffer a direct-to-LDS copy is still filling, and would make every LDS read
// wait for all outstanding copies (copy latency and matrix work then add up instead of overlapping).
// So these reads are issued as opaque instructions on LDS byte addresses and waited for explicitly;
// the wait names the registers it protects, which orders their consumers after it.
typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef __attribute__((address_space(3))) float lds_f32;
__device__ __forceinline__ unsigned lds_addr(const lds_u8* p) { return (unsigned)(__UINTPTR_TYPE__)p; }
__device__ __forceinline__ bf16x8 lds_frag(const lds_u8* p) {
  const u32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(p);
  return __builtin_bit_cast(bf16x8, v);
}
__device__ __forceinline__ bf16x8 lds_frag_raw(unsigned addr) {
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
__device__ __forceinline__ void lds_wait(bf16x8& a, bf16x8& b, bf16x8& c, bf16x8& d) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d)::"memory");
}
__device__ __forceinline__ void lds_wait(bf16x8& a, bf16x8& b, bf16x8& c) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b), "+v"(c)::"memory");
}
__device__ __forceinline__ void lds_wait(bf16x8& a, bf16x8& b) {
  asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b)::"memory");
}
// LDS transpose read (gfx950): within each block of 16 lanes, lane i receives element i % 4 of the 8 bytes that
// lanes i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12 of the block address.  With lane s of a block pointing at row
// k0 + s / 4, columns n0 + 4 (s % 4) .. + 3 of a row-major bf16 tile, lane i gets column n0 + i of rows k0 .. k0 + 3:
// an operand fragment along the tile's rows, read from a tile stored along its columns.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x2 lds_tr16_raw(unsigned addr) {
  u32x2 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v) : "v"(addr) : "memory");
  return v;
}
__device__ __forceinline__ void lds_wait(u32x2& a, u32x2& b) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b)::"memory"); }
// the same, leaving the newest KEEP LDS requests of this wave in flight
template <int KEEP>
__device__ __forceinline__ void lds_wait_keep(bf16x8& a, bf16x8& b, bf16x8& c, bf16x8& d) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(KEEP) : "memory");
}
template <int KEEP>
__device__ __forceinline__ void lds_wait_keep(bf16x8& a, bf16x8& b, bf16x8& c) {
  asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(a), "+v"(b), "+v"(c) : "n"(KEEP) : "memory");
}

// Barrier of the role loops: LDS traffic of this wave is complete, global loads / copies stay in flight
// (__syncthreads() would also drain every outstanding global access, and with it the prefetches).
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// asynchronous global -> LDS copy of `bytes` (a multiple of NW KB) shared by the NW matrix-core waves of a workgroup
template <int NW = 8>
__device__ __forceinline__ void dma_copy(const char* src, lds_u8* dst, int bytes, int mw, int lane) {
  for (int k = mw; k < bytes / 1024; k += NW)
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + k * 1024 + lane * 16),
                                     (__attribute__((address_space(3))) void*)(dst + k * 1024), 16, 0, 0);
}

}  // namespace
}  // namespace adapm
