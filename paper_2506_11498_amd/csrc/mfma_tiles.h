// Building blocks of the bf16 MFMA attention kernels (gfx950): 32x32x16 MFMA wrappers, the
// swizzled row-major LDS tile that every operand is staged in, and its two read patterns.
//
// MFMA v_mfma_f32_32x32x16_bf16, lane l (l32 = l % 32, g = l / 32):
//   A operand: row l32,  k-slots 8g .. 8g+7        B operand: column l32, k-slots 8g .. 8g+7
//   C/D:       column l32, 16 floats i -> row 8*(i/4) + 4g + i%4
//
// A tile is [rows][128 bf16] = 256 bytes per row = 16 chunks of 16 bytes; chunk c of row r is
// stored at chunk c ^ swz(r).  swz is a bijection on 16 consecutive rows (row-pattern reads of
// 16 lanes hit 16 different chunks) and moves rows r, r+1, r+2, r+3 to different 64-byte units
// (transposed reads of 4 rows x 32 bytes spread over the banks).
#pragma once
#include "common.h"

namespace lrsa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int TILE_ROW_BYTES = 256;  // head_dim 128 in bf16

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }

// byte offset of chunk `c` (16 bytes) of row `r`
__device__ __forceinline__ int tile_off(int r, int c) { return r * TILE_ROW_BYTES + ((c ^ swz(r)) << 4); }

// Operand with the tile's rows as MFMA rows/columns and head_dim as the contraction:
// lane takes row rb + l32, channels 16*kk + 8g .. +7  (one 16-byte LDS read).
__device__ __forceinline__ bf16x8 read_rows(const unsigned char* tile, int rb, int kk, int l32, int g) {
    return *reinterpret_cast<const bf16x8*>(tile + tile_off(rb + l32, kk * 2 + g));
}

// Operand with head_dim as MFMA rows and 16 tile rows as the contraction ("transposed" read):
// lane takes channel db*32 + l32 and the 8 k-slots of its half g, where slot j is tile row
// rb16 + 8*(j/4) + 4g + j%4 -- exactly the rows a C-layout accumulator hands over when its
// registers 8h .. 8h+7 are reused as the other operand.
// ds_read_b64_tr_b16 works per 16-lane group: lane i receives, as element e, element i%4 of the
// 8 bytes that lane 4e + i/4 of its group points at.  So source lane lam points at row
// 4g + lam/4 (+8 for the second read), channels dbase + 4*(lam%4) .. +3.
__device__ __forceinline__ bf16x8 read_cols(const unsigned char* tile, int rb16, int db, int lane) {
    const int lam = lane & 15, m = (lane >> 4) & 1, g = lane >> 5;
    const int ch = db * 32 + 16 * m + 4 * (lam & 3);  // first channel of the 8 bytes this lane points at
    const int r0 = rb16 + 4 * g + (lam >> 2);
    const int c = ch >> 3, within = (ch & 7) * 2;
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(tile + tile_off(r0, c) + within));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(tile + tile_off(r0 + 8, c) + within));
    union { s16x4 h[2]; bf16x8 v; } u;
    u.h[0] = lo;
    u.h[1] = hi;
    return u.v;
}

// Per-lane byte offsets of the two read patterns inside a tile.  Because the swizzle is an XOR on
// chunk bits that the channel-block index also occupies, the offset of channel block kk (or db, and of
// the second transposing read) is the block-0 offset XOR a compile-time constant: two registers per
// lane describe every read, other row blocks (multiples of 16 rows) are immediates on top.
struct LaneOffs {
    int row;   // read_rows: row l32, channel block 0
    int col;   // read_cols: channel block 0, first transposing read
};
__device__ __forceinline__ LaneOffs make_lane_offs(int lane) {
    LaneOffs o;
    const int l32 = lane & 31, g = lane >> 5, lam = lane & 15, m = (lane >> 4) & 1;
    o.row = tile_off(l32, g);
    const int ch = 16 * m + 4 * (lam & 3);
    o.col = tile_off(4 * g + (lam >> 2), ch >> 3) + (ch & 7) * 2;
    return o;
}
// same operands as read_rows / read_cols; rb is a multiple of 32, rb16 of 16
__device__ __forceinline__ bf16x8 read_rows_o(const unsigned char* tile, const LaneOffs& o, int rb, int kk) {
    return *reinterpret_cast<const bf16x8*>(tile + (o.row ^ (kk << 5)) + rb * TILE_ROW_BYTES);
}
__device__ __forceinline__ bf16x8 read_cols_o(const unsigned char* tile, const LaneOffs& o, int rb16, int db) {
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(tile + (o.col ^ (db << 6)) + rb16 * TILE_ROW_BYTES));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_ptr)(tile + (o.col ^ ((db << 6) | 32)) + (rb16 + 8) * TILE_ROW_BYTES));
    union { s16x4 h[2]; bf16x8 v; } u;
    u.h[0] = lo;
    u.h[1] = hi;
    return u.v;
}

// The same two reads with the tile's LDS address already folded into the lane's offset register (one add
// per tile instead of one per read): valid when the tile starts on a 256-byte boundary, because XORing a
// constant below 256 then commutes with adding the base.  rows16 is a compile-time row offset (multiple of 16).
typedef bf16x8 __attribute__((address_space(3))) * lds_bf16x8_ptr;
__device__ __forceinline__ unsigned lds_addr(const void* p) {
    return (unsigned)(size_t)(__attribute__((address_space(3))) void*)p;
}
__device__ __forceinline__ bf16x8 read_rows_a(unsigned arow, int kk) {
    return *(lds_bf16x8_ptr)(size_t)(arow ^ unsigned(kk << 5));
}
__device__ __forceinline__ bf16x8 read_cols_a(unsigned acol, int rows16, int db) {
    typedef s16x4 __attribute__((address_space(3))) * lds_ptr;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(size_t)((acol ^ unsigned(db << 6)) + rows16 * TILE_ROW_BYTES));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_ptr)(size_t)((acol ^ unsigned((db << 6) | 32)) + (rows16 + 8) * TILE_ROW_BYTES));
    union { s16x4 h[2]; bf16x8 v; } u;
    u.h[0] = lo;
    u.h[1] = hi;
    return u.v;
}

// registers i0 .. i0+7 of a C-layout accumulator as a bf16 operand
__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int i0) {
    f32x8 t;
#pragma unroll
    for (int j = 0; j < 8; ++j) t[j] = v[i0 + j];
    return __builtin_convertvector(t, bf16x8);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- asynchronous global -> LDS copies (global_load_lds_dwordx4) --------------------------------
// One wave instruction moves 64 x 16 bytes: lane l's 16 bytes land at lds_base + 16*l (checked on the
// hardware), i.e. four consecutive 256-byte tile rows starting at row r4.  The swizzle is applied on
// the global side: the lane whose slot is physical chunk pc of row r fetches logical chunk pc ^ swz(r).
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void gbl_void_t;

// tile row and 16-byte logical chunk this lane fetches when its wave fills rows r4 .. r4+3
__device__ __forceinline__ int async_row(int r4, int lane) { return r4 + (lane >> 4); }
__device__ __forceinline__ int async_chunk(int row, int lane) { return (lane & 15) ^ swz(row); }

// The copies are issued through inline assembly, so the compiler does not know that LDS is written
// behind its back: it would otherwise make LDS reads of OTHER ring stages wait for all copies in flight
// (its alias bookkeeping for such copies is limited).  Ordering is the kernels' own business: they wait
// with wait_vmcnt<n>() for the copies of the stage they are about to read and synchronise the workgroup.
// Hidden operations are harmless for the compiler's own vmcnt arithmetic: vector memory loads complete in
// order, so "at most n outstanding" still implies that everything it knows to be older has arrived.
// M0 (the LDS base of the copy) is saved and restored around the instruction.
__device__ __forceinline__ void async_copy16(const void* src, const void* lds_dst) {
    const unsigned la = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lds_void_t*)lds_dst);   // wave-uniform
    unsigned keep;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(src), "s"(la)
        : "memory");
}
__device__ __forceinline__ void async_copy4(const void* src, const void* lds_dst) {
    const unsigned la = __builtin_amdgcn_readfirstlane((unsigned)(size_t)(lds_void_t*)lds_dst);
    unsigned keep;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %1, off\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(src), "s"(la)
        : "memory");
}
// The same copy with the global address given as a wave-uniform base (scalar registers) plus this lane's unsigned
// 32-bit byte offset, and the LDS destination as a wave-uniform byte address: no 64-bit vector arithmetic and no
// pointer conversion per copy.  The caller guarantees offsets below 4 GiB.
__device__ __forceinline__ void async_copy16_so(const void* base, unsigned voff, unsigned lds_byte_addr) {
    unsigned keep;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(voff), "s"(base), "s"(lds_byte_addr)
        : "memory");
}
// ... and with a per-lane 64-bit global address (rows that come from two different buffers)
__device__ __forceinline__ void async_copy16_la(const void* src, unsigned lds_byte_addr) {
    unsigned keep;
    asm volatile(
        "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
        : "=&s"(keep)
        : "v"(src), "s"(lds_byte_addr)
        : "memory");
}
// src: this lane's 16 bytes in global memory; tile: LDS tile base; r4: first of the 4 rows (wave-uniform)
__device__ __forceinline__ void async_rows4(const void* src, unsigned char* tile, int r4) {
    async_copy16(src, tile + r4 * TILE_ROW_BYTES);
}

// s_waitcnt vmcnt(0) in the form the compiler understands: every vector memory load it has issued so far
// (Q fragments and the like) is complete afterwards, so it will not place waits of its own for them inside
// the ring loop, where they would also drain the asynchronous copies.
__device__ __forceinline__ void wait_all_vmem_known() { __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8)); }

// Pins a loaded register operand at this point of the program: the empty volatile statement "uses and
// redefines" it, so the load that produced it cannot be moved below (volatile statements keep their order,
// and the asynchronous copies are such statements) and later uses carry no pending-load bookkeeping.
template <class T>
__device__ __forceinline__ void pin_loaded(T& v) {
    asm volatile("" : "+v"(v));
}

// s_waitcnt vmcnt(n) alone
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Scalar-cache load of one 32-bit word at a wave-uniform address, issued explicitly (the compiler only
// picks the scalar path for memory it can prove unwritten, which the asynchronous copies defeat).  The
// result may be used only after smem_wait() on the same variables.
__device__ __forceinline__ int smem_load(const int32_t* base, int index) {
    int v;
    const int off = __builtin_amdgcn_readfirstlane(index * 4);
    asm volatile("s_load_dword %0, %1, %2" : "=s"(v) : "s"(base), "s"(off) : "memory");
    return v;
}
// eight scalars (no array: indexing a private array invites the compiler to move it to memory)
struct Scalar8 { int a0, a1, a2, a3, a4, a5, a6, a7; };
// waits for all outstanding scalar loads (and LDS reads); ties the 8 values to the wait (they are scalar
// registers already: the loads' outputs)
__device__ __forceinline__ void smem_wait(Scalar8& v) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+s"(v.a0), "+s"(v.a1), "+s"(v.a2), "+s"(v.a3), "+s"(v.a4), "+s"(v.a5), "+s"(v.a6), "+s"(v.a7)
                 :
                 : "memory");
}
// the one of four scalars that belongs to this lane's quarter q4 = lane / 16 (three conditional moves)
__device__ __forceinline__ int pick4(int q4, int x0, int x1, int x2, int x3) {
    int r = x0;
    r = q4 == 1 ? x1 : r;
    r = q4 == 2 ? x2 : r;
    r = q4 == 3 ? x3 : r;
    return r;
}

// Workgroup barrier without the memory fence of __syncthreads(): the fence would make the compiler wait
// for ALL outstanding vector memory operations, i.e. also for the asynchronous copies of later ring
// stages.  The caller has already waited (wait_vmcnt) for exactly the copies that must have landed; LDS
// reads of the stage about to be refilled have been consumed by MFMAs before the wave gets here.  The
// "memory" clobber keeps the compiler from moving LDS accesses across the barrier.
__device__ __forceinline__ void ring_barrier() { asm volatile("s_barrier" ::: "memory"); }

// position of stream entry j: the gather list (sink positions, then the flattened survivor
// lists) followed by the contiguous window that starts at cs
__device__ __forceinline__ int stream_pos(const Dims& D, const int32_t* idx_h, int j, int ng, int cs) {
    if (j < ng) return j < D.S ? j : idx_h[j - D.S];
    return cs + (j - ng);
}

// Which (batch, KV head, head subset, query tile) a workgroup of a query-outer kernel takes.
// per_unit = workgroups per (batch, KV head).  With xcd_map, consecutive workgroup ids -- which the
// hardware deals round-robin to the 8 XCDs -- belong to 8 different KV heads, so that one XCD's L2
// keeps serving the K/V rows of the same head.
struct QTileMap {
    int sink_tiles, tpc, tiles;   // query tiles of QT rows: in the sink, per chunk, per head
    int tix_lo, tix_hi;           // the tiles that are launched (all of them unless a row window is set)
    int gsubs, per_unit, xcd_map;
};
__device__ __forceinline__ void decode_qtile(const QTileMap& M, const Dims& D, int i, int& b, int& h, int& gsub,
                                             int& tix) {
    int unit, w;
    if (M.xcd_map) {
        const int j = i >> 3;
        unit = (i & 7) + 8 * (j / M.per_unit);
        w = j % M.per_unit;
    } else {
        unit = i / M.per_unit;
        w = i % M.per_unit;
    }
    b = unit / D.Hkv;
    h = unit % D.Hkv;
    gsub = w % M.gsubs;
    tix = M.tix_hi - 1 - w / M.gsubs;   // heaviest (latest) query tile first
}

// ---- condensed KV cache --------------------------------------------------------------------------
// Kc, Vc [B, Hkv, gl, 128] bf16, contiguous: row j of a head is the K (V) row of entry j of its gather list
// (sink tokens, then the survivors chunk by chunk); gl = S + K * Ns.
inline int gather_list_len(const Dims& D) { return D.nq > 0 ? D.S + D.K * D.Ns : 0; }
inline size_t compact_kv_bytes(const Dims& D) {
    return D.compact ? 2 * align256(size_t(D.B) * D.Hkv * gather_list_len(D) * 128 * sizeof(bf16_t)) : 0;
}
hipError_t launch_compact_kv(const Dims& D, const void* K, const void* V, const int32_t* idx, void* Kc, void* Vc,
                             hipStream_t st);
// address of the row of stream entry j (gather list, then the contiguous window) with a condensed cache
__device__ __forceinline__ const bf16_t* stream_row(const bf16_t* Zc, const bf16_t* Z, int64_t stride, int j, int ng,
                                                    int cs) {
    return j < ng ? Zc + int64_t(j) * 128 : Z + int64_t(cs + (j - ng)) * stride;
}

// heads of a group that share a workgroup: the largest of 4, 2, 1 that divides the group size
inline int heads_per_wg(const Dims& D) { return D.G % 4 == 0 ? 4 : D.G % 2 == 0 ? 2 : 1; }

inline QTileMap make_qtile_map(const Dims& D, int gh, int waves) {
    QTileMap M;
    const int qt = 32 * (waves / gh);
    const int sink_rows = D.S < D.n ? D.S : D.n;
    M.sink_tiles = (sink_rows + qt - 1) / qt;
    M.tpc = (D.L + qt - 1) / qt;
    M.tiles = M.sink_tiles + D.nq * M.tpc;
    M.tix_lo = D.row_begin == 0 ? 0 : M.sink_tiles + D.fq0 * M.tpc;
    M.tix_hi = M.sink_tiles + D.fq1 * M.tpc;
    M.gsubs = D.G / gh;
    M.per_unit = (M.tix_hi - M.tix_lo) * M.gsubs;
    M.xcd_map = (D.B * D.Hkv) % 8 == 0 ? 1 : 0;
    return M;
}

}  // namespace lrsa
