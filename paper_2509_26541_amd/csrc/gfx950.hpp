// Small pieces shared by the gfx950 kernels of this library: vector types, a compile-time loop, the
// direct global->LDS load and the workgroup-to-XCD remap.
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

namespace tasp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

// One direct global->LDS load of 16 bytes per lane (global_load_lds_dwordx4): lane l reads
// base + off and its bytes land at lds_base + 16 l, so the 64 lanes of a wavefront fill 1 KiB of
// consecutive LDS.  No registers and no LDS write instruction are involved; it counts in vmcnt only.
// The compiler does not see it as a memory operation: the caller waits (s_waitcnt vmcnt) and
// publishes the data with a barrier before anybody reads it.  FENCE adds a compiler-level memory
// clobber for callers whose LDS reads are ordinary loads the compiler could otherwise move across.
// m0 is written here without being declared: the compiler reserves it (it never keeps a value
// there, and names it only immediately before an instruction that reads it).
template <bool FENCE>
__device__ inline void global_to_lds_16(const unsigned char* base, unsigned off, unsigned char* lds_base) {
  const unsigned lds_addr = static_cast<unsigned>(reinterpret_cast<size_t>((lds_void_ptr)lds_base));
  if constexpr (FENCE)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(off), "s"(base) : "memory");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(off), "s"(base));
}

// Four bytes per lane: lane l's dword lands at lds_base + 4 l (a gather of 64 scalars into one
// 256-byte row of LDS, with no register in between).
template <bool FENCE>
__device__ inline void global_to_lds_4(const unsigned char* base, unsigned off, unsigned char* lds_base) {
  const unsigned lds_addr = static_cast<unsigned>(reinterpret_cast<size_t>((lds_void_ptr)lds_base));
  if constexpr (FENCE)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(lds_addr), "v"(off), "s"(base) : "memory");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(lds_addr), "v"(off), "s"(base));
}

// The same load through a buffer descriptor: lane l reads descriptor base + soff + off, where soff
// is a scalar register.  A gather whose lanes share a moving base then needs no vector arithmetic
// at all: the base moves in soff.  Raw descriptor (no stride, no swizzle), 2^32 - 1 records, so
// every offset sum below 2^32 - 4 is in range; offsets are unsigned 32-bit, like the form above.
__device__ inline u32x4 raw_buffer(const void* base) {
  const unsigned long long b = reinterpret_cast<unsigned long long>(base);
  u32x4 r;
  r[0] = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(b)));
  r[1] = static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(b >> 32))) & 0xffffu;   // 48-bit address, stride 0
  r[2] = 0xffffffffu;
  r[3] = 0x00020000u;          // 32-bit data format, raw buffer
  return r;
}
template <bool FENCE = false>
__device__ inline void buffer_to_lds_16(const u32x4& rsrc, unsigned soff, unsigned off, unsigned char* lds_base) {
  const unsigned lds_addr = static_cast<unsigned>(reinterpret_cast<size_t>((lds_void_ptr)lds_base));
  if constexpr (FENCE)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" : : "s"(lds_addr), "v"(off), "s"(rsrc), "s"(soff) : "memory");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" : : "s"(lds_addr), "v"(off), "s"(rsrc), "s"(soff));
}

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2); this maps the hardware
// index to a work index such that every XCD gets one contiguous run of the work list.
__device__ inline int xcd_contiguous(int block, int nblocks) {
  const int xcd = block & 7, slot = block >> 3;
  const int q8 = nblocks >> 3, r8 = nblocks & 7;
  return xcd * q8 + (xcd < r8 ? xcd : r8) + slot;
}

// The same for a work list that is `units` runs of `per_unit` items, a unit being what reads the
// same K and V (one KV head of one sequence), each run sorted by falling work.  When the units do
// not divide among the 8 XCDs, equal counts per XCD are not equal work (half a run is its longer
// or its shorter items) and an XCD whose run ends with the long items of a part-unit finishes late.
// So 8/g XCDs (g = gcd(units, 8)) share units/g units and deal their items round-robin: every one of
// them gets the same mix and still meets each unit's items by falling work.  With units a multiple
// of 8 this is xcd_contiguous.  The grid has xcd_balanced_blocks workgroups; -1 = none for this one.
__host__ __device__ inline int xcd_balanced_share(int units) { const int g = units & -units; return g >= 8 ? 1 : 8 / g; }
__device__ inline int xcd_balanced(int block, int units, int per_unit) {
  const int k = xcd_balanced_share(units);
  const int xcd = block & 7, slot = block >> 3;
  const int len = units / (8 / k) * per_unit;          // items of a group of k XCDs
  const int j = slot * k + xcd % k;
  return j < len ? xcd / k * len + j : -1;
}
__host__ inline long long xcd_balanced_blocks(long long units, long long per_unit) {
  const long long k = xcd_balanced_share(static_cast<int>(units));
  const long long len = units / (8 / k) * per_unit;
  return 8 * ((len + k - 1) / k);
}

// Work item of persistent workgroup `block` (of `nblocks`, a multiple of 8 and fewer than
// n_items) in its `round`-th turn, or -1 when it has none left.  XCD x owns the same contiguous run
// of items as in xcd_contiguous, and its nblocks/8 workgroups walk that run in rounds, forwards in
// even rounds and backwards in odd ones, so that a run sorted by falling work is shared out evenly.
__device__ inline int persistent_item(int block, int nblocks, int n_items, int round) {
  const int xcd = block & 7, slot = block >> 3, slots = nblocks >> 3;
  const int q8 = n_items >> 3, r8 = n_items & 7;
  const int start = xcd * q8 + (xcd < r8 ? xcd : r8), cnt = q8 + (xcd < r8 ? 1 : 0);
  const int pos = round * slots + ((round & 1) ? slots - 1 - slot : slot);
  return pos < cnt ? start + pos : -1;
}

}  // namespace tasp
