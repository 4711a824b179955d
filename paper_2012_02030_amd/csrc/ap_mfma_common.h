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

// One swizzle that serves both kinds of read, for tiles that are read row-wise and through the
// transposing load: a bijection on r % 16 (r % 8 for D = 64, (r / 4) % 4 for D = 32) as the
// row-wise reads need, whose upper chunk bits follow the low row bits as the transposing reads need.
template <int D> __device__ __forceinline__ int swz_u(int r)
{
    return D == 128 ? (((r & 3) << 2) | ((r >> 2) & 3))
                    : (D == 64 ? ((((r >> 1) & 1) << 2) | ((r >> 2) & 3)) : ((r >> 2) & 3));
}
enum { SWZ_KEY = 0, SWZ_VALUE = 1, SWZ_BOTH = 2 };
template <int D, int S> __device__ __forceinline__ int swz(int r)
{
    return S == SWZ_KEY ? swz_k<D>(r) : (S == SWZ_VALUE ? swz_v<D>(r) : swz_u<D>(r));
}

// two floats -> two bf16 (round to nearest even) in one register: the hardware conversion, one
// instruction per pair
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack_bf16_rne(float lo, float hi)
{
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}
// The same rounding in integer arithmetic (finite inputs).  Used where a kernel sits at its
// register limit: the compiler converts several pairs ahead of their stores with the form above,
// and in the layout-walking dK/dV kernel at D = 128 that costs a spilled register.
__device__ __forceinline__ uint32_t pack_bf16_rne_int(float lo, float hi)
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
// M0 is listed as clobbered so that no value of the compiler's own is assumed to survive in it.
typedef __attribute__((ext_vector_type(4))) int rsrc_t;
__device__ __forceinline__ void load16_to_lds(unsigned lds_addr, int voff, rsrc_t rsrc, int soff)
{
    // the descriptor and the scalar offset are wave-uniform by construction; say so where the
    // compiler cannot see it (values that went through memory or a loop), else it picks VGPRs
    rsrc.x = __builtin_amdgcn_readfirstlane(rsrc.x);
    rsrc.y = __builtin_amdgcn_readfirstlane(rsrc.y);
    rsrc.z = __builtin_amdgcn_readfirstlane(rsrc.z);
    rsrc.w = __builtin_amdgcn_readfirstlane(rsrc.w);
    soff = __builtin_amdgcn_readfirstlane(soff);
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
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

// N such loads in a row, as one instruction sequence: load u puts 1 KB at lds_addr + u * LSTEP
// and reads at per-lane offset voff[u] plus scalar offset soff + u * sstep.  M0 and the scalar
// offset advance by one scalar addition each between two loads (the second one also provides the
// wait state that a write of M0 needs before the next LDS-direct load), so a load costs three
// instructions and no vector arithmetic.
#define AP_DMA_LD(v) "buffer_load_dwordx4 %[" v "], %[rs], %[t] offen lds\n\t"
#define AP_DMA_NX "s_add_u32 m0, m0, %[ls]\n\ts_add_u32 %[t], %[t], %[ss]\n\t"
#define AP_DMA_HEAD "s_mov_b32 m0, %[lds]\n\ts_mov_b32 %[t], %[so]\n\t"
template <int N, int LSTEP>
__device__ __forceinline__ void load16_chain(unsigned lds_addr, int soff, int sstep, const int* voff, rsrc_t rsrc)
{
    static_assert(N == 1 || N == 2 || N == 4 || N == 8, "loads per wavefront, operand and tile");
    rsrc.x = __builtin_amdgcn_readfirstlane(rsrc.x);         // wave-uniform by construction, see above
    rsrc.y = __builtin_amdgcn_readfirstlane(rsrc.y);
    rsrc.z = __builtin_amdgcn_readfirstlane(rsrc.z);
    rsrc.w = __builtin_amdgcn_readfirstlane(rsrc.w);
    soff = __builtin_amdgcn_readfirstlane(soff);
    sstep = __builtin_amdgcn_readfirstlane(sstep);
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    int t;
    if constexpr (N == 1)
        asm volatile(AP_DMA_HEAD AP_DMA_LD("v0")
                     : [t] "=&s"(t)
                     : [lds] "s"(lds_addr), [so] "s"(soff), [rs] "s"(rsrc), [v0] "v"(voff[0])
                     : "memory", "m0");
    else if constexpr (N == 2)
        asm volatile(AP_DMA_HEAD AP_DMA_LD("v0") AP_DMA_NX AP_DMA_LD("v1")
                     : [t] "=&s"(t)
                     : [lds] "s"(lds_addr), [so] "s"(soff), [ss] "s"(sstep), [ls] "n"(LSTEP), [rs] "s"(rsrc),
                       [v0] "v"(voff[0]), [v1] "v"(voff[1])
                     : "memory", "m0", "scc");
    else if constexpr (N == 4)
        asm volatile(AP_DMA_HEAD AP_DMA_LD("v0") AP_DMA_NX AP_DMA_LD("v1") AP_DMA_NX AP_DMA_LD("v2")
                         AP_DMA_NX AP_DMA_LD("v3")
                     : [t] "=&s"(t)
                     : [lds] "s"(lds_addr), [so] "s"(soff), [ss] "s"(sstep), [ls] "n"(LSTEP), [rs] "s"(rsrc),
                       [v0] "v"(voff[0]), [v1] "v"(voff[1]), [v2] "v"(voff[2]), [v3] "v"(voff[3])
                     : "memory", "m0", "scc");
    else
        asm volatile(AP_DMA_HEAD AP_DMA_LD("v0") AP_DMA_NX AP_DMA_LD("v1") AP_DMA_NX AP_DMA_LD("v2")
                         AP_DMA_NX AP_DMA_LD("v3") AP_DMA_NX AP_DMA_LD("v4") AP_DMA_NX AP_DMA_LD("v5")
                             AP_DMA_NX AP_DMA_LD("v6") AP_DMA_NX AP_DMA_LD("v7")
                     : [t] "=&s"(t)
                     : [lds] "s"(lds_addr), [so] "s"(soff), [ss] "s"(sstep), [ls] "n"(LSTEP), [rs] "s"(rsrc),
                       [v0] "v"(voff[0]), [v1] "v"(voff[1]), [v2] "v"(voff[2]), [v3] "v"(voff[3]),
                       [v4] "v"(voff[4]), [v5] "v"(voff[5]), [v6] "v"(voff[6]), [v7] "v"(voff[7])
                     : "memory", "m0", "scc");
}
#undef AP_DMA_LD
#undef AP_DMA_NX
#undef AP_DMA_HEAD

// The swizzle of the row that lane l handles in load instruction j repeats in j with this period
// (swz_k and swz_u of a D = 128 tile see 4 rows per instruction and repeat every 16 rows, ...).
template <int D, int S> constexpr int swz_period() { return S == SWZ_VALUE ? 1 : (D == 128 ? 4 : (D == 64 ? 2 : 1)); }
constexpr int const_gcd(int a, int b) { return b == 0 ? a : const_gcd(b, a % b); }

// Issue the loads of one 64-row tile (rows row0.. of a [rows, D] bf16 slice described by the
// buffer resource) into LDS with swizzle S (SWZ_KEY, SWZ_VALUE or SWZ_BOTH).  Every wavefront
// instruction moves 64 x 16 bytes = 1 KB; wavefront w issues instructions w, w + NW, ...
template <int D, int NW, int S>
__device__ __forceinline__ void issue_tile_loads(rsrc_t rsrc, lds_u16* dst, int row0,
                                                 int stride_bytes, int wave, int lane)
{
    constexpr int CPR = D / 8;                // 16-byte chunks per row
    constexpr int RPI = 64 / CPR;             // rows per wavefront instruction
    constexpr int NI = kBN / RPI;             // instructions per tile
    static_assert(NI % NW == 0, "instructions must divide over the wavefronts");
    constexpr int N = NI / NW;
    constexpr int PU = swz_period<D, S>() / const_gcd(swz_period<D, S>(), NW);   // period in u
    const int rl = lane / CPR;                // row inside the instruction
    const int cp = lane % CPR;                // chunk position in LDS
    int voff[N];
#pragma unroll
    for (int u = 0; u < N; ++u) {
        const int r = (wave + NW * (u % PU)) * RPI + rl;      // a row with the swizzle of load u's
        voff[u] = rl * stride_bytes + (cp ^ swz<D, S>(r)) * 16;
    }
    load16_chain<N, NW * 1024>(lds_addr_of(dst + wave * 512), (row0 + wave * RPI) * stride_bytes,
                               NW * RPI * stride_bytes, voff, rsrc);
}

// Same for a gathered entry: row u of this lane's instructions comes from key gidx[u]
// (an empty slot holds Lk, which lies beyond num_records and reads as zeros).  Keys and the
// row stride in bytes are below 2^24 (checked by the host), so the full-rate 24-bit multiply serves.
template <int D, int NW, int S>
__device__ __forceinline__ void issue_gather_loads(rsrc_t rsrc, lds_u16* dst, const int* gidx,
                                                   int stride_bytes, int wave, int lane)
{
    constexpr int CPR = D / 8;
    constexpr int RPI = 64 / CPR;
    constexpr int NI = kBN / RPI;
    constexpr int N = NI / NW;
    constexpr int PU = swz_period<D, S>() / const_gcd(swz_period<D, S>(), NW);
    const int rl = lane / CPR;
    const int cp = lane % CPR;
    int voff[N];
#pragma unroll
    for (int u = 0; u < N; ++u) {
        const int r = (wave + NW * (u % PU)) * RPI + rl;
        voff[u] = (int)__umul24((unsigned)gidx[u], (unsigned)stride_bytes) + (cp ^ swz<D, S>(r)) * 16;
    }
    load16_chain<N, NW * 1024>(lds_addr_of(dst + wave * 512), 0, 0, voff, rsrc);
}

// C[64 x 32] = T[64 x D] * R^T[D x 32]: T is a 64-row tile in LDS (rows of D bf16, key swizzle),
// R^T the operand this wavefront keeps in registers (lane l: row l % 32 of R, elements
// 16*kk + 8*(l/32) .. +7).  Result in the matrix-core layout: lane l holds column l % 32 and,
// of each 32-row block, rows 8*(i/4) + 4*(l/32) + i%4.  n = l % 32, k_swz = (l / 32) ^ swz_k(n).
template <int D>
__device__ __forceinline__ void qk_64(const uint16_t* Ks, const bf16x8* qreg, int n, int k_swz,
                                      f32x16* sacc)
{
    constexpr int KSTEPS = D / 16;
    constexpr int AHEAD = KSTEPS < 3 ? KSTEPS : 3;           // key operands requested this many steps early
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[kb][i] = 0.f;
    bf16x8 kreg[KSTEPS][2];
    auto read_step = [&](int kk) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
            kreg[kk][kb] = *reinterpret_cast<const bf16x8*>(Ks + (kb * 32 + n) * D + ((2 * kk) ^ k_swz) * 8);
    };
#pragma unroll
    for (int kk = 0; kk < AHEAD; ++kk) read_step(kk);
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        if (kk + AHEAD < KSTEPS) read_step(kk + AHEAD);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
            sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kreg[kk][kb], qreg[kk], sacc[kb], 0, 0, 0);
    }
    // pin that order, so that LDS latency is paid once per tile and not once per step
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * AHEAD, 0);
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        if (kk + AHEAD < KSTEPS) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
    }
}

// Makes the compiler place its own wait for these loaded registers here (right after a
// wait_vmem(), where it costs nothing) instead of in front of their first real use, where it
// would also wait for the tile loads issued in between.
template <int N>
__device__ __forceinline__ void settle(bf16x8* q)
{
#pragma unroll
    for (int kk = 0; kk < N; ++kk) asm volatile("" : "+v"(q[kk]));
}

// Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  This bijection gives
// every XCD one contiguous range of the linear workgroup index, so that the workgroups that
// share the K and Q rows of a head (and example) also share an L2.
__device__ __forceinline__ int xcd_contiguous(int bid, int grid)
{
    const int x = bid & 7, q = grid >> 3, r = grid & 7;
    return x * q + min(x, r) + (bid >> 3);
}

// One 512-byte block (64 x 8 bytes, or 128 x 4 bytes) into LDS by the first 32 lanes of a wavefront.
__device__ __forceinline__ void dma_512(lds_u16* dst, const void* src_base, unsigned src_bytes, long long byte_off,
                                        int lane)
{
    if (lane < 32) {
        const rsrc_t rs = make_rsrc(src_base, src_bytes);
        load16_to_lds(lds_addr_of(dst), lane * 16, rs, (int)byte_off);
    }
}

// Per-lane constants of the transposing LDS reads of a 64-row tile stored with the value swizzle.
struct TrRead {
    int lane_row, in_chunk, chunk_lo, swz;
};
template <int D>
__device__ __forceinline__ TrRead make_tr_read(int lane)
{
    const int hh = lane >> 5, i16 = lane & 15, g = (lane >> 4) & 1, vj = i16 >> 2;
    TrRead t;
    t.lane_row = 4 * hh + vj;
    t.in_chunk = 4 * (i16 & 1);
    t.chunk_lo = 2 * g + ((i16 >> 1) & 1);
    t.swz = swz_v<D>(vj) >> 2;                               // xor on the 4-chunk group index
    return t;
}

// acc^T[D x 32] += T^T[D x 64] * P[64 x 32]: T is a 64-row tile in LDS (value swizzle), read with
// the transposing load; P is held in the layout qk_64 produces (fp32, rounded to bf16 here).
// The operands of 16-row step ks + 1 are requested before the matrix instructions of step ks.
template <int D>
__device__ __forceinline__ void tr_mm_64(lds_u16* Ts, const f32x16* p, f32x16* acc, const TrRead& t)
{
    constexpr int DBLK = D / 32;
    auto read_t = [&](int ks, bf16x8* treg) {
#pragma unroll
        for (int db = 0; db < DBLK; ++db) {
            const int chunk = ((db ^ t.swz) << 2) + t.chunk_lo;
            lds_u16* p0 = Ts + (16 * ks + t.lane_row) * D + chunk * 8 + t.in_chunk;
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p0);
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0 + 8 * D));
            treg[db] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    bf16x8 tcur[DBLK], tnext[DBLK];
    read_t(0, tcur);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[e] = (__bf16)p[ks >> 1][8 * (ks & 1) + e];
        if (ks + 1 < 4) read_t(ks + 1, tnext);
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
            acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tcur[db], pb, acc[db], 0, 0, 0);
#pragma unroll
        for (int db = 0; db < DBLK; ++db) tcur[db] = tnext[db];
    }
}

// The same product for a tile stored with the swizzle SWZ_BOTH.
template <int D>
struct TrReadU {
    int off[2][D / 32];      // element offsets of this lane's two reads of every 32-column block
};
template <int D>
__device__ __forceinline__ TrReadU<D> make_tr_read_u(int lane)
{
    const int hh = lane >> 5, i16 = lane & 15, g = (lane >> 4) & 1, vj = i16 >> 2;
    const int lane_row = 4 * hh + vj, in_chunk = 4 * (i16 & 1), chunk_lo = 2 * g + ((i16 >> 1) & 1);
    const int fx = swz_u<D>(lane_row);                       // row + 8 flips bit 1 of the swizzle
    TrReadU<D> t;
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
        t.off[0][db] = lane_row * D + ((4 * db + chunk_lo) ^ fx) * 8 + in_chunk;
        t.off[1][db] = (lane_row + 8) * D + ((4 * db + chunk_lo) ^ fx ^ 2) * 8 + in_chunk;
    }
    return t;
}
template <int D>
__device__ __forceinline__ void tr_mm_64_u(lds_u16* Ts, const f32x16* p, f32x16* acc, const TrReadU<D>& t)
{
    constexpr int DBLK = D / 32;
    auto read_t = [&](int ks, bf16x8* treg) {
#pragma unroll
        for (int db = 0; db < DBLK; ++db) {
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(Ts + 16 * ks * D + t.off[0][db]));
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(Ts + 16 * ks * D + t.off[1][db]));
            treg[db] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    bf16x8 tcur[DBLK], tnext[DBLK];
    read_t(0, tcur);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        bf16x8 pb;
#pragma unroll
        for (int e = 0; e < 8; ++e) pb[e] = (__bf16)p[ks >> 1][8 * (ks & 1) + e];
        if (ks + 1 < 4) read_t(ks + 1, tnext);
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
            acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tcur[db], pb, acc[db], 0, 0, 0);
#pragma unroll
        for (int db = 0; db < DBLK; ++db) tcur[db] = tnext[db];
    }
}

// Write acc^T[D x 32] * mul as 32 bf16 rows of D elements: staged through this wavefront's own
// 32 x D region of LDS (key swizzle), then 128-bit stores; rows >= rows_valid are dropped.
template <int D>
__device__ __forceinline__ void store_rows_bf16(uint16_t* stage, const f32x16* acc, float mul, int lane,
                                                uint16_t* dst, long long row_stride, int rows_valid)
{
    constexpr int DBLK = D / 32, CPR = D / 8;
    const int n = lane & 31, hh = lane >> 5;
    const int f = swz_k<D>(n);
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            uint2 w;
            w.x = pack_bf16_rne_int(acc[db][4 * g4] * mul, acc[db][4 * g4 + 1] * mul);
            w.y = pack_bf16_rne_int(acc[db][4 * g4 + 2] * mul, acc[db][4 * g4 + 3] * mul);
            const int chunk = (4 * db + g4) ^ f;
            *reinterpret_cast<uint2*>(stage + n * D + chunk * 8 + 4 * hh) = w;
        }
    // the same wavefront reads back what it wrote: no barrier needed, only LDS ordering
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int u = 0; u < (32 * CPR) / 64; ++u) {
        const int idx = u * 64 + lane;
        const int rr = idx / CPR, c = idx % CPR;
        const uint4 v = *reinterpret_cast<const uint4*>(stage + rr * D + (c ^ swz_k<D>(rr)) * 8);
        if (rr < rows_valid) *reinterpret_cast<uint4*>(dst + (size_t)rr * row_stride + c * 8) = v;
    }
}

}  // namespace mfma
}  // namespace ap
