// Device helpers shared by the bf16 MFMA kernels (dgrad in gemm_bf16.hip, wgrad in wgrad_bf16.hip):
// fragment types, the LDS-direct load, buffer descriptors, tile orders.
#pragma once

#include <type_traits>

#include "groups.hpp"

namespace vcas {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2v;
typedef __attribute__((ext_vector_type(2))) float f32x2v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int BK = 64;  // contraction elements per step

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2v v = {lo, hi};
    bf16x2v r = __builtin_convertvector(v, bf16x2v);
    return *reinterpret_cast<uint32_t *>(&r);
}

// All global reads of the GEMMs are raw buffer loads: a 128-bit resource descriptor in SGPRs
// (base, size), a per-thread byte offset in one VGPR, the loop's advance in an SGPR.  Reads past
// the end of the tensor return zero, so a masked-out row is just an offset beyond the end
// (kOutside) and ragged tails need no branches.
constexpr uint32_t kOutside = 0x80000000u;   // tensors are < 2 GiB (checked on the host)

// slot XOR of row k of a [k][columns] tile: the four k rows that a half-wave transposes at once
// (ds_read_b64_tr_b16) land in four different 64-byte bank groups
__device__ __forceinline__ int wswz(int k) { return (k & 3) * 4; }

// 128-bit buffer descriptor built by hand (base, stride 0, size in bytes, raw dword format) for
// use in inline assembly.
__device__ __forceinline__ i32x4 raw_descriptor(const void *base, uint32_t bytes)
{
    const uint64_t b = reinterpret_cast<uint64_t>(base);
    i32x4 d;
    d[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    d[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((b >> 32) & 0xffffu));
    d[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    d[3] = 0x00020000;
    return d;
}

// One LDS-direct load: every lane fetches 16 bytes at buffer offset voffset + soffset, the
// wavefront's 1 KiB lands at LDS byte address lds_base (wave-uniform) in lane order.  Written as
// assembly so that the compiler does not track it: it would otherwise make every later LDS read
// wait for ALL loads in flight (it cannot tell the stages apart), and the waits are placed by
// hand before the barrier anyway.
__device__ __forceinline__ void lds_direct_load16(i32x4 desc, uint32_t lds_base, uint32_t voffset, uint32_t soffset)
{
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_base), "v"(voffset), "s"(desc), "s"(soffset)
                 : "memory", "m0");
}

// Row of the 32x32 accumulator block that register v of this lane holds; the column is lane % 32.
__device__ __forceinline__ int acc_row(int v) { return (v >> 2) * 8 + ((threadIdx.x & 63) >> 5) * 4 + (v & 3); }

// XCD-aware tile order: consecutive workgroup ids land on different XCDs (id mod 8), so hand each
// XCD one contiguous run of tiles; neighbours in the run share operand rows through that XCD's L2.
__device__ __forceinline__ int xcd_remap(int id, int total)
{
    const int per = (total + 7) / 8;
    return (id & 7) * per + (id >> 3);
}

// Tile number -> (row tile, column tile), column panels of panel_w tiles, row-major inside a panel.
__device__ __forceinline__ void panel_order_rt(int tile, int tiles_m, int tiles_n, int panel_w, int &tile_m,
                                               int &tile_n)
{
    const int panel = tile / (tiles_m * panel_w);
    const int in_panel = tile - panel * tiles_m * panel_w;
    const int width = min(panel_w, tiles_n - panel * panel_w);
    tile_m = in_panel / width;
    tile_n = panel * panel_w + in_panel % width;
}

template <typename Kern>
static bool allow_lds(Kern kern, size_t bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)bytes) == hipSuccess;
}

}  // namespace vcas
