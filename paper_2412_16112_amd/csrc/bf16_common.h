// Device-side building blocks shared by the bf16 kernels (forward and backward) for gfx950, head_dim
// CLEAR_HEAD_DIM (128 unless the including file sets 64):
// vector types, the LDS layout of a staged 64-token tile and its swizzle, LDS-direct staging loads, MFMA
// operand reads from a staged tile (row-wise and transposed), the element masks of Eq. 3, and the two
// 32 x 32 block products every kernel is made of.
#pragma once
#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>
#include <utility>

#include "block_class.h"
#include "clear_internal.h"

namespace clear {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#ifndef CLEAR_HEAD_DIM
#define CLEAR_HEAD_DIM 128
#endif
constexpr int D = CLEAR_HEAD_DIM;    // head_dim
static_assert(D == 128 || D == 64, "row layout, swizzle and operand addresses are worked out for 128 and 64 channels");
constexpr int KS = D / 16;           // contraction steps of Q K^T (16 channels per matrix instruction)
constexpr int NDB = D / 32;          // 32-channel slices of O
constexpr int CHUNKS = D / 8;        // 16-byte chunks per token row
constexpr int ROW_BYTES = D * 2;     // one token row of K or V
constexpr int ROWS_PER_LOAD = 1024 / ROW_BYTES;  // token rows one LDS-direct wave load covers
constexpr int TILE_KEYS = kKeyTileKeys;
constexpr int TILE_BYTES = TILE_KEYS * ROW_BYTES;  // 16 KB for K, same for V
// How many matrix instructions ahead the forward tile pipeline reads its LDS operands.  At 128 channels the image-query
// kernel sits at its 168-register limit (three waves per SIMD with the loading waves): with two slots ahead, and the
// fourth operand buffer that needs, the compiler keeps a query fragment in scratch memory and reloads it inside every
// tile (a 16-byte scratch load and a full wait in front of a matrix instruction; 4 % of the kernel's time), with one
// slot ahead nothing in the tile loops is spilled.  64 channels have the registers for two.
#ifndef CLEAR_OPERAND_PREFETCH
#if CLEAR_HEAD_DIM == 128
#define CLEAR_OPERAND_PREFETCH 1
#else
#define CLEAR_OPERAND_PREFETCH 2
#endif
#endif
#ifndef CLEAR_TILES_PER_STAGE
#define CLEAR_TILES_PER_STAGE 2
#endif
constexpr int TPS = CLEAR_TILES_PER_STAGE;           // key tiles (K + V = 32 KB each) staged per barrier
#ifndef CLEAR_NBUF
#define CLEAR_NBUF 2
#endif
constexpr int NBUF = CLEAR_NBUF;                     // stage buffers: one being computed on, the others being filled
__host__ __device__ constexpr int next_buf(int buf) { return buf + 1 == NBUF ? 0 : buf + 1; }
constexpr int STAGE_BYTES = TPS * 2 * TILE_BYTES;
constexpr float FAST_SUM_LIMIT = 1.0e30f;  // the fast pass is discarded when a query's sums leave [0, 1e30)
constexpr float M_INIT = -1.0e30f;         // finite "no key seen yet" (keeps exp2 arguments free of inf - inf)

// LDS layout of a staged tile: 64 rows of ROW_BYTES, unpadded (the LDS-direct load writes 1 KB per wave
// instruction), with the 16-byte chunks of each row permuted: logical chunk c of row k sits in slot
// c ^ swz(k).
// 256-byte rows (a row = one sweep over the banks): swz is a bijection on 16 consecutive rows (the 32 key
// rows of a K read spread over all banks) and sends 4 consecutive rows to 4 different 64-byte quads (so does
// the transposed V read).
// 128-byte rows (two rows per sweep): on the even rows of 16 consecutive rows swz is a bijection onto the 8
// chunks (K read), and rows k and k + 2, which share a half sweep, land in different 64-byte quads (V read).
// Both have period 16 in the row.
__host__ __device__ constexpr int swz(int row)
{
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | (((row >> 3) & 1) << 1) | ((row >> 2) & 1));
}

__device__ __forceinline__ float wave_pair_max(float x)
{
    // lanes l and l ^ 32 hold the two halves of one query's scores
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

__device__ __forceinline__ float wave_pair_sum(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// One 16-byte-per-lane load from global memory straight into LDS: the wave writes 1 KB starting at
// lds_addr (wave-uniform), lane i at lds_addr + 16 i; lane i reads gbase + voff.  Counted by vmcnt.
// Written as asm so that the compiler does not serialise later LDS reads behind it; the kernel waits
// with explicit s_waitcnt vmcnt before the barrier that publishes the tile.
__device__ __forceinline__ void load_to_lds_16B(const void* gbase, unsigned voff, unsigned lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(gbase) : "memory", "m0");
}

// This lane's index in its wave from the hardware's lane count (two instructions, no register kept live for it).
__device__ __forceinline__ int fresh_lane_id()
{
    int l;
    asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
    return l;
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));  // expcnt, lgkmcnt unconstrained
}

// Query/key prologue on 8 consecutive channels (4 rotary pairs) of one token, in fp32: RMS-norm gain, then
// the rotation by the sum of the row angle and the column angle (tables hold (cos, sin) per pair).
// g0, g1: this chunk's 8 gains; a0, a1 / b0, b1: its 8 floats of the token's row / column table rows.
__device__ __forceinline__ void prologue_chunk_values(float (&x)[8], float inv_rms, bool has_gain, const f32x4& g0, const f32x4& g1,
                                                      bool turn, const f32x4& a0, const f32x4& a1, const f32x4& b0, const f32x4& b1)
{
    if (has_gain) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[j] = x[j] * inv_rms * g0[j];
            x[4 + j] = x[4 + j] * inv_rms * g1[j];
        }
    }
    if (turn) {
        const float cy[4] = {a0[0], a0[2], a1[0], a1[2]}, sy[4] = {a0[1], a0[3], a1[1], a1[3]};
        const float cx[4] = {b0[0], b0[2], b1[0], b1[2]}, sx[4] = {b0[1], b0[3], b1[1], b1[3]};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const float c = cy[t] * cx[t] - sy[t] * sx[t];
            const float s = sy[t] * cx[t] + cy[t] * sx[t];
            const float e = x[2 * t], o = x[2 * t + 1];
            x[2 * t] = c * e - s * o;
            x[2 * t + 1] = s * e + c * o;
        }
    }
}
// The same, fetching the chunk's table entries: gain8 / ry8 / rx8 point at its 8 floats of the gain vector and
// of the token's two table rows (null: that step is skipped).
__device__ __forceinline__ void prologue_chunk(float (&x)[8], float inv_rms, const float* gain8, const float* ry8, const float* rx8)
{
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 g0 = zero, g1 = zero, a0 = zero, a1 = zero, b0 = zero, b1 = zero;
    if (gain8) {
        g0 = *(const f32x4*)gain8;
        g1 = *(const f32x4*)(gain8 + 4);
    }
    if (ry8) {
        a0 = *(const f32x4*)ry8;
        a1 = *(const f32x4*)(ry8 + 4);
        b0 = *(const f32x4*)rx8;
        b1 = *(const f32x4*)(rx8 + 4);
    }
    prologue_chunk_values(x, inv_rms, gain8 != nullptr, g0, g1, ry8 != nullptr, a0, a1, b0, b1);
}

struct WaveState {
    f32x16 oacc[NDB];  // O^T tiles: channel 32*db + 8*(reg/4) + 4*hh + reg%4 of this lane's query
    float m_run;     // running maximum, raw logits (may lag the true maximum by < 2^8 in the exponent)
    float l_run;     // this lane's share of the denominator
    float c;         // log2(e) / sqrt(head_dim)
};

// Per-lane LDS read offsets inside a staged tile.  All operand addresses of a tile derive from two
// offsets by XOR with small constants and by adding multiples of 4 KB (ds_read immediates):
//   K operand, block blk, contraction step ks:  ((tile + k0) ^ (ks << 5)) + blk * 32 rows
//   V operand, block blk, step s2, slice db:    ((tile + TILE_BYTES + v0 [^ V_HI]) ^ (db << 6)) + blk * 32 rows + s2 * 16 rows
// (tile addresses are multiples of 1 KB, so the XORs stay inside the offsets' own bits).
struct LaneOffsets {
    unsigned k0;  // row qi, logical chunk hh:  qi * ROW_BYTES + ((hh ^ swz(qi)) << 4)
    unsigned v0;  // transpose read, slice 0, first half of the 16-key step
};
// second half of the step: key rows + 8 (8 * ROW_BYTES) and what that does to their swizzle (chunk bit 1 either way)
constexpr unsigned V_HI = (1u << 5) | (unsigned)(8 * ROW_BYTES);

// Lane addresses of one staged tile (LDS byte addresses).
struct TileAddr {
    unsigned kb, vb0, vb1;
};
// (v_half: where in the staged tile the half that is read transposed starts; the forward kernels read K row-wise
// from the first half and V transposed from the second)
__device__ __forceinline__ TileAddr tile_addr(unsigned tile_lds, const LaneOffsets& lo, unsigned v_half = TILE_BYTES)
{
    TileAddr ta;
    ta.kb = tile_lds + lo.k0;
    ta.vb0 = tile_lds + v_half + lo.v0;
    ta.vb1 = tile_lds + v_half + (lo.v0 ^ V_HI);
    return ta;
}

enum MaskMode : int { kMaskNone = 0, kMaskLinear = 1, kMaskImage = 2, kMaskTable = 3 };

// Which family of image masks a kernel instance is compiled for.  The disc of Eq. 3 is the product path and
// gets a kernel of its own, so that the code of the compared masks (integer divisions per element for the
// Swin windows, strided token addresses) neither lengthens it nor shares its instruction cache.
enum MaskCode : int { kCodeDisc = 0, kCodeGeneric = 1, kCodeFull = 2 };
__host__ __device__ constexpr int mask_code_of(int mask_kind)
{
    return mask_kind == kMaskDisc ? kCodeDisc : (mask_kind == kMaskFull ? kCodeFull : kCodeGeneric);
}

// Read-only tables (tile lists, lane masks) are addressed through the constant address space so that
// they are fetched with scalar loads: wave-uniform, and not counted among the vector loads whose
// completion the tile prefetch waits on.
typedef const __attribute__((address_space(4))) int* const_int_ptr;
typedef const __attribute__((address_space(4))) unsigned long long* const_u64_ptr;

struct MaskArgs {
    int a, b;  // linear: first token of the tile, token limit; image: tile origin (row, col)
    int hh, qy, qx, gridH, gridW, r2;
    int kind, r, shift;    // MaskKind; for kinds other than the disc: radius / window size and Swin shift
    const_u64_ptr row[2];  // kMaskTable: 16 lane masks per key block (one per score register)
};

// Sets the scores of inadmissible (query, key) pairs of key block kb to -inf.  Register r of this lane
// is key slot 8*(r/4) + 4*hh + r%4 of the block (Eq. 3 for image keys; the token limit for linear tiles).
template <int MASK, int CODE>
__device__ __forceinline__ void apply_mask(f32x16& s, int kb, const MaskArgs& ma)
{
    if (MASK == kMaskTable) {
        // precomputed per relative block offset: bit l of row[r] says whether lane l keeps score register r
        const_u64_ptr row = ma.row[kb & 1];  // wave-uniform address: the words are read into scalar registers
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = __builtin_amdgcn_inverse_ballot_w64(row[r]) ? s[r] : -INFINITY;
    } else if (MASK == kMaskLinear) {
        const int base = ma.a + 32 * kb + 4 * ma.hh;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            if (base + 8 * (r >> 2) + (r & 3) >= ma.b) s[r] = -INFINITY;
    } else if (MASK == kMaskImage && CODE != kCodeDisc) {
        // The other local masks.  Square and Swin windows are products of a row condition and a column condition:
        // 4 + 4 tests per block instead of 16 pair tests (kCodeFull: only the grid's edge).
        const int ky0 = ma.a + kKeyBlockH * kb, kx0 = ma.b + 4 * ma.hh;
        bool row_ok[4], col_ok[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int ky = ky0 + g, kx = kx0 + g;
            row_ok[g] = ky < ma.gridH && (CODE == kCodeFull || axis_admits(ma.kind, ma.r, ma.shift, ma.qy, ky));
            col_ok[g] = kx < ma.gridW && (CODE == kCodeFull || axis_admits(ma.kind, ma.r, ma.shift, ma.qx, kx));
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const bool keep = row_ok[e >> 2] && col_ok[e & 3];
            s[e] = keep ? s[e] : -INFINITY;
        }
    } else if (MASK == kMaskImage) {
        const int ky0 = ma.a + kKeyBlockH * kb, kx0 = ma.b + 4 * ma.hh;
        int dx2[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int dx = kx0 + t - ma.qx;
            dx2[t] = (kx0 + t < ma.gridW) ? dx * dx : 0x7fffffff;  // columns beyond the grid never pass
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int dy = ky0 + g - ma.qy;
            const int lim = (ky0 + g < ma.gridH) ? ma.r2 - dy * dy : 0;  // dx^2 must stay below lim
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (!(dx2[t] < lim)) s[4 * g + t] = -INFINITY;
        }
    }
}

// p = 2^{(s - m) c} for the 16 scores of one block; returns their sum; packs them as the B operand of P V.
__device__ __forceinline__ float exp_block(const f32x16& s, float c, float mc, bf16x8 (&pf)[2])
{
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], c, -mc));
        sum += pv;
        pf[r >> 3][r & 7] = (__bf16)pv;
    }
    return sum;
}

__device__ __forceinline__ float max_block(const f32x16& s)
{
    float mx = fmaxf(s[0], s[1]);
#pragma unroll
    for (int r = 2; r < 16; ++r) mx = fmaxf(mx, s[r]);
    return mx;
}

// Scheduling hints: ask the backend to emit, in this order, `n` instructions of the given class.
// Classes (LLVM AMDGPU sched_group_barrier masks): 0x2 VALU, 0x8 MFMA, 0x100 LDS read.
#define SCHED_GROUP(mask, n) __builtin_amdgcn_sched_group_barrier((mask), (n), 0)

typedef const __attribute__((address_space(3))) bf16x8* lds_bf16x8_ptr;
typedef __attribute__((address_space(3))) short4v* lds_short4_ptr;

// (extra: a constant byte offset on top, e.g. TILE_BYTES for the second half of a staged tile, so that both halves
// share the lane's swizzled addresses and differ in the instruction's immediate offset only)
__device__ __forceinline__ bf16x8 read_k_operand(const TileAddr& ta, int blk, int ks, unsigned extra = 0)
{
    return *(lds_bf16x8_ptr)(size_t)((ta.kb ^ (unsigned)(ks << 5)) + (unsigned)(blk * 32 * ROW_BYTES) + extra);
}

// V^T fragment for the contraction over key slots 16 s2 + 4 hh + {0..3} and 16 s2 + 8 + 4 hh + {0..3} of
// block blk, channels 32 db .. 32 db + 31: two 16-bit transpose reads.
__device__ __forceinline__ bf16x8 read_v_operand(const TileAddr& ta, int blk, int s2, int db, unsigned extra = 0)
{
    const unsigned imm = (unsigned)(blk * 32 * ROW_BYTES + s2 * 16 * ROW_BYTES) + extra;
    const short4v lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(size_t)((ta.vb0 ^ (unsigned)(db << 6)) + imm));
    const short4v hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(size_t)((ta.vb1 ^ (unsigned)(db << 6)) + imm));
    union { struct { short4v lo, hi; } h; bf16x8 v; } u;
    u.h.lo = lo4;
    u.h.hi = hi4;
    return u.v;
}

__device__ __forceinline__ f32x16 qk_block(const TileAddr& ta, int blk, const bf16x8 (&qf)[KS], unsigned extra = 0)
{
    f32x16 s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_k_operand(ta, blk, ks, extra), qf[ks], s, 0, 0, 0);
    return s;
}

// O^T += V_blk^T P^T for one 32-key block.  The contraction step s2 pairs P registers 8*s2 .. 8*s2+7
// with key slots 16*s2 + 4*hh + {0..3} and 16*s2 + 8 + 4*hh + {0..3}.
__device__ __forceinline__ void pv_block(f32x16 (&oacc)[NDB], const TileAddr& ta, int blk, const bf16x8 (&pf)[2], unsigned extra = 0)
{
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
            oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_v_operand(ta, blk, s2, db, extra), pf[s2], oacc[db], 0, 0, 0);
}

// Raises a kernel's dynamic-LDS limit once per device (function attributes belong to the device's copy of the
// kernel), safely from several host threads: one slot per kernel instantiation, which the caller keeps in a
// function-local static.
struct LdsLimitOnce {
    static constexpr int kDevices = 64;
    std::once_flag once[kDevices];
    hipError_t result[kDevices] = {};
    hipError_t ensure(const void* kernel, int bytes)
    {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kDevices) return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        std::call_once(once[dev], [&] { result[dev] = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); });
        return result[dev];
    }
};

// Pins the instruction order: nothing is scheduled across this point.
#define SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// f(integral_constant<int, 0>{}), ..., f(integral_constant<int, N - 1>{}), in order.
template <typename F, int... Is>
__device__ __forceinline__ void static_for_impl(F& f, std::integer_sequence<int, Is...>)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

}  // namespace
}  // namespace clear
