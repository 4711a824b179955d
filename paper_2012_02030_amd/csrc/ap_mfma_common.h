// Device helpers shared by the matrix-core kernels (attention forward, attention-map
// accumulation): vector types, LDS swizzles, LDS-direct tile loads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ap {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) uint16_t lds_u16;

constexpr int kBN = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLazy = 8.0f;   // log2 of the largest P before the softmax reference is raised

// Swizzles: the 16-byte chunk c of LDS row r is stored at chunk position c ^ f(r).
// Key rows are read as one chunk per lane by 32 consecutive rows; value rows are read by the
// transposing load, 8 rows x 64 bytes per wavefront instruction.
template <int D> __device__ __forceinline__ int swz_k(int r) { return (r * (D / 8) / 16) % (D / 8); }
template <int D> __device__ __forceinline__ int swz_v(int r)
{
    return D == 128 ? 4 * (r & 3) : (D == 64 ? 4 * ((r >> 1) & 1) : 0);
}

__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi)
{
    uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
    a += 0x7fffu + ((a >> 16) & 1u);
    b += 0x7fffu + ((b >> 16) & 1u);
    return (a >> 16) | (b & 0xffff0000u);
}

__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// One 128-bit buffer load per lane whose data goes straight to LDS: lane l's 16 bytes land at
// lds_addr + 16*l.  lds_addr (a byte address, wave-uniform) travels in M0.  The instruction is
// written as inline assembly on purpose: the compiler then does not know that LDS is being
// written asynchronously, so it does not make every later LDS read wait for all loads in
// flight; completion is enforced by wait_vmem() and the workgroup barrier in the main loop.
typedef __attribute__((ext_vector_type(4))) int rsrc_t;
__device__ __forceinline__ void load16_to_lds(unsigned lds_addr, int voff, rsrc_t rsrc, int soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}

// Raw buffer descriptor: base address, stride 0, num_records bytes; loads beyond num_records
// return zeros.
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, unsigned num_bytes)
{
    rsrc_t r;
    r.x = (int)(uintptr_t)base;
    r.y = (int)(((uintptr_t)base >> 32) & 0xffffu);
    r.z = (int)num_bytes;
    r.w = 0x00020000;
    return r;
}

__device__ __forceinline__ unsigned lds_addr_of(lds_u16* p) { return (unsigned)(uintptr_t)p; }

// Issue the loads of one 64-row tile (rows row0.. of a [rows, D] bf16 slice described by the
// buffer resource) into LDS.  Every wavefront instruction moves 64 x 16 bytes = 1 KB.
template <int D, int NW, bool IS_V>
__device__ __forceinline__ void issue_tile_loads(rsrc_t rsrc, lds_u16* dst, int row0,
                                                 int stride_bytes, int wave, int lane)
{
    constexpr int CPR = D / 8;                // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;             // rows per wavefront instruction
    constexpr int NI = kBN / RPI;             // instructions per tile
    static_assert(NI % NW == 0, "instructions must divide over the wavefronts");
    const int rl = lane / CPR;                // row inside the instruction
    const int cp = lane % CPR;                // chunk position in LDS
#pragma unroll
    for (int u = 0; u < NI / NW; ++u) {
        const int j = wave + NW * u;
        const int r = j * RPI + rl;           // row inside the tile
        const int c = cp ^ (IS_V ? swz_v<D>(r) : swz_k<D>(r));
        const int voff = rl * stride_bytes + c * 16;
        const int soff = (row0 + j * RPI) * stride_bytes;
        load16_to_lds(lds_addr_of(dst + j * 512), voff, rsrc, soff);
    }
}

// Same for a gathered entry: row u of this lane's instructions comes from key gidx[u]
// (an empty slot holds Lk, which lies beyond num_records and reads as zeros).
template <int D, int NW, bool IS_V>
__device__ __forceinline__ void issue_gather_loads(rsrc_t rsrc, lds_u16* dst, const int* gidx,
                                                   int stride_bytes, int wave, int lane)
{
    constexpr int CPR = D / 8;
    constexpr int RPI = 64 / CPR;
    constexpr int NI = kBN / RPI;
    const int rl = lane / CPR;
    const int cp = lane % CPR;
#pragma unroll
    for (int u = 0; u < NI / NW; ++u) {
        const int j = wave + NW * u;
        const int r = j * RPI + rl;
        const int c = cp ^ (IS_V ? swz_v<D>(r) : swz_k<D>(r));
        const int voff = gidx[u] * stride_bytes + c * 16;
        load16_to_lds(lds_addr_of(dst + j * 512), voff, rsrc, 0);
    }
}

}  // namespace mfma
}  // namespace ap
