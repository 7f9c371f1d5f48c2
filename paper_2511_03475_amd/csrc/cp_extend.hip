// cp_extend: prefix-cached "extend" prefill attention over a paged KV cache for gfx950.
//
// Kernels behind the C ABI of cp_extend.h:
//   write_kv_kernel       cache append (paper, Section 1: the prefix cache stores prior K/V)
//   extend_attn_kernel    suffix rows attend to cached prefix pages + their own K/V
//                         (paper, Section 1 / Section 2.1: prefill over a prefix cache)
//   decode_attn_kernel    the same for calls with few rows per KV head (a wavefront per key chunk)
//   merge_splits_kernel, merge_few_splits_kernel   combine partial results over key ranges
//   check_tables_kernel   optional check of block_table against the pool size
//
// Attention kernel layout.  One workgroup = 8 wavefronts = 256 query rows of one q head; each
// wavefront owns 32 rows.  Keys are streamed in tiles of 64 through LDS.  Scores are computed
// transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16 so that the accumulator lane
// (lane % 32) is a query row: the softmax row reductions are then in-lane plus one exchange
// between the two half-waves, the bf16 probabilities already sit in the B-operand layout of the
// second product O^T = V^T P^T, and the per-row rescale of O is a per-lane scalar multiply.
// V^T fragments come from LDS through the transposing read ds_read_b64_tr_b16.  The K/V tiles
// reach LDS by direct loads (global_load_lds_dwordx4), without a pass through registers.  The
// query fragments carry softmax_scale * log2(e), rounded to bf16 once per row, so that the
// accumulators of S^T are the arguments of exp2 as they stand.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <algorithm>
#include <atomic>
#include <mutex>
#include <type_traits>
#include <vector>

#include "cp_extend.h"

namespace {

constexpr int kD = 128;       // head dim
constexpr int kPS = 16;       // tokens per page
constexpr int kBM = 256;      // query rows per workgroup
constexpr int kBN = 64;       // keys per tile
constexpr int kThreads = 512; // 8 wavefronts
constexpr int kXcds = 8;      // accelerator complex dies; workgroup ids round-robin over them
constexpr int kMaxSplits = 64;
constexpr int kWaves = kThreads / 64;
constexpr int kNKB = kBN / 32;            // 32-key blocks per tile
constexpr int kLoadRows = kWaves * 4;     // key rows one load step of the workgroup covers
static_assert(kBM == kWaves * 32 && kBN == 2 * kLoadRows, "tile shape");

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

struct AttnParams {
    const uint16_t *q;
    const uint16_t *k_new;
    const uint16_t *v_new;
    const uint16_t *kv_pages;
    const int32_t *block_table;
    const int32_t *prefix_lens;
    const int32_t *extend_lens;
    uint16_t *out;
    float *part_o;  // [nsplit][T][Hq][D]   unnormalised partial outputs
    float *part_ml; // [nsplit][T][Hq][2]   running max (log2 domain) and sum
    int32_t batch, Hq, Hkv, G, max_pages, T;
    int32_t nsplit;
    int32_t dec_row_blocks; // decode kernel: blocks of 32 (head, token) rows per (request, KV head)
    int32_t items_per_head; // work units per KV head * nsplit
    int32_t total_items;    // items_per_head * Hkv
    int32_t items_per_xcd;  // ceil(total_items / 8)
    float scale_log2;       // softmax_scale * log2(e)
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Maximum across the two half-waves (lane l and lane l ^ 32 end with the same value).
__device__ __forceinline__ float halfwave_max(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halfwave_sum(float x)
{
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Number of q heads of one KV head that share a workgroup (GQA head sharing): short extends
// leave most of a 256-row tile empty, so the rows of up to 8 heads are packed into it.  The
// largest power of two that divides G and still gives every head enough rows for E.
__host__ __device__ inline int heads_per_tile(int E, int G)
{
    int pack = 1;
    while (pack < 8 && (G & (2 * pack - 1)) == 0 && E * (pack * 2) <= kBM) pack *= 2;
    return pack;
}
// Work units (row tiles x head groups) of one request for one KV head; pack = heads_per_tile.
__host__ __device__ inline int units_of_request(int E, int G, int pack)
{
    if (E <= 0) return 0;
    int shift = 0;
    while ((1 << shift) < pack) ++shift;
    return ((E * pack + kBM - 1) / kBM) * (G >> shift);
}
// Inclusive prefix sum over the 64 lanes of a wavefront.
__device__ __forceinline__ int wave_inclusive_scan(int x, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(x, off, 64);
        if (lane >= off) x += y;
    }
    return x;
}

// LDS: four K buffers and five V buffers of one 64-key tile (16 KiB) each, K of tile t in buffer
// t % 4, V in buffer t % 5.  A tile is requested two iterations before its first use and V(t) is
// still read one iteration after K(t).  The workgroup meets at a barrier only after every second
// tile (tiles 2m+1 and 2m+2 form an interval): within an interval K(2m+1), K(2m+2), V(2m) and
// V(2m+1) are read, V(2m+2) is resident, and tiles 2m+3 and 2m+4 arrive, which takes four K
// buffers and five V buffers if no arriving tile is to overwrite one that a slower wavefront of
// the same interval still reads.
// The tiles come from global memory straight into LDS (global_load_lds_dwordx4: lane i of a
// wavefront writes 16 bytes at slot i of 1 KiB, no way through registers and no LDS store
// instruction), so rows cannot be padded: they are 256 bytes apart and the 16-byte chunks
// inside a row are swizzled instead.  K: chunk c of row r sits at slot c ^ (r & 15) (16
// consecutive rows at the same column fall into 16 different 16-byte bank groups); V: at slot
// c ^ ((r & 3) << 2) (the four consecutive rows of a transposing read fall into four different
// 64-byte bank groups).
constexpr int kNumBufs = 4;
constexpr int kPitchK = 256;
constexpr int kPitchV = 256;
constexpr int kTileBytesK = kBN * kPitchK;
constexpr int kTileBytesV = kBN * kPitchV;
constexpr int kNumBufsV = 5;
constexpr int kLdsBytes = kNumBufs * kTileBytesK + kNumBufsV * kTileBytesV;

template <bool kSplit>
__global__ __launch_bounds__(kThreads) void extend_attn_kernel(const AttnParams p)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    char *const lds_k = lds;                          // [4][64 rows][256 B]
    char *const lds_v = lds + kNumBufs * kTileBytesK; // [5][64 rows][256 B]

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int j = lane & 31; // query row within the wave; also key row / d row of A operands
    const int h = lane >> 5; // half-wave

    // ---- which work item: consecutive workgroup ids land on different XCDs, so give each
    // XCD a contiguous range of the item list (one KV head per XCD when Hkv == 8) and keep the
    // items that stream the same K/V next to each other in time.
    const int bid = blockIdx.x;
    const int vid = (bid % kXcds) * p.items_per_xcd + bid / kXcds;
    if (vid >= p.total_items) return;
    const int kvh = vid / p.items_per_head;
    int rem = vid - kvh * p.items_per_head;
    const int split = rem % p.nsplit;
    int unit = rem / p.nsplit;

    // Units of a KV head: requests in order; within a request the last (longest) row tile
    // first, and for each row tile the groups of q heads that are packed into one workgroup.
    // The request that owns the unit is found 64 requests at a time: every lane takes one
    // request, a prefix sum over the wavefront gives the first unit of each (a sequential scan
    // costs a dependent scalar load and several integer divisions per request, ~1.5 us each).
    int r = p.batch, cu = 0, E = 0, t = 0, pack = 1, hgroup = 0;
    for (int base = 0; base < p.batch; base += 64) {
        const int rr = base + lane;
        const int e_l = rr < p.batch ? p.extend_lens[rr] : 0;
        const int units_l = units_of_request(e_l, p.G, heads_per_tile(e_l, p.G));
        const int incl_u = wave_inclusive_scan(units_l, lane);
        const int incl_e = wave_inclusive_scan(e_l, lane);
        const int total_u = __builtin_amdgcn_readlane(incl_u, 63);
        if (unit < total_u) {
            const int first = __builtin_ctzll(__builtin_amdgcn_ballot_w64(incl_u > unit));
            r = base + first;
            unit -= __builtin_amdgcn_readlane(incl_u - units_l, first);
            cu += __builtin_amdgcn_readlane(incl_e - e_l, first);
            E = __builtin_amdgcn_readlane(e_l, first);
            break;
        }
        unit -= total_u;
        cu += __builtin_amdgcn_readlane(incl_e, 63);
    }
    if (r < p.batch) {
        pack = heads_per_tile(E, p.G);
        int shift = 0;
        while ((1 << shift) < pack) ++shift;
        const int groups = p.G >> shift;
        const int nt = (E * pack + kBM - 1) / kBM; // row tiles of kBM / pack rows
        hgroup = unit % groups;
        t = nt - 1 - unit / groups;
    }
    if (r >= p.batch) return;
    const int P = p.prefix_lens[r];

    // GQA head sharing: `pack` q heads of the KV head share the workgroup's K/V tiles, each
    // with kBM / pack query rows; a wavefront belongs to exactly one of them.
    const int rows_per_head = kBM / pack;
    const int head = kvh * p.G + hgroup * pack + (wave * 32) / rows_per_head;
    const int q0 = t * rows_per_head;                          // first extend row of the tile
    const int wave_row0 = q0 + (wave * 32) % rows_per_head;    // first row of this wavefront
    const int row_i = wave_row0 + j;                           // this lane's extend row (may be >= E)
    const int rows_end = min(E, q0 + rows_per_head);           // one past the last valid row
    const int np_tiles = (P + kBN - 1) / kBN;        // prefix key tiles
    const int ns_tiles = (rows_end + kBN - 1) / kBN; // suffix key tiles up to the diagonal
    const int n_tiles = np_tiles + ns_tiles;
    const int per_split = (n_tiles + p.nsplit - 1) / p.nsplit;
    const int kt_begin = split * per_split;
    const int kt_end = min(n_tiles, kt_begin + per_split);
    const int n_it = kt_end - kt_begin;              // key tiles of this work item

    const int64_t out_row = (int64_t)(cu + min(row_i, E - 1));
    const bool row_valid = row_i < E;

    if (n_it <= 0) {
        // empty split: the merge skips entries whose sum is zero
        if (kSplit && row_valid && h == 0) {
            float *ml = p.part_ml + (((int64_t)split * p.T + out_row) * p.Hq + head) * 2;
            ml[0] = -INFINITY;
            ml[1] = 0.f;
        }
        return;
    }

    // ---- Q fragments, B operand of S^T = K Q^T: lane (j, h) holds q[row j][16 kk + 8 h ..+8)
    // The fragments hold q * softmax_scale * log2(e), rounded to bf16 (nearest even) once per
    // row: the accumulators of S^T are then the arguments of exp2 as they stand, which saves one
    // multiply-add per score (a third of the softmax instructions).  The rounding moves every
    // query element by at most half a bf16 unit in the last place.
    const float c = p.scale_log2;
    bf16x8 qf[8];
    {
        const uint16_t *qp = p.q + (out_row * p.Hq + head) * kD + 8 * h;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const bf16x8 raw = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(qp + 16 * kk));
#pragma unroll
            for (int e = 0; e < 8; ++e) qf[kk][e] = (__bf16)((float)raw[e] * c);
        }
    }

    // ---- this thread's share of a K/V tile: key rows ld_row and ld_row + kLoadRows, 16-byte chunk
    // ld_chunk.  The four rows a wavefront loads per step share one page, so the block-table
    // lookup and the page base are scalar; rows past the end of the prefix (or of the suffix)
    // re-read the last valid row so that no uninitialised cache slot is ever touched.
    const int ld_sub = lane >> 4;         // row within the wavefront's group of four
    const int ld_row = wave * 4 + ld_sub; // 0..kLoadRows-1
    const int ld_chunk = lane & 15;
    // read-only for the whole launch and every index is wavefront-uniform: the constant address
    // space keeps these loads on the scalar unit although the direct loads below write memory
    const __attribute__((address_space(4))) int32_t *table =
        (const __attribute__((address_space(4))) int32_t *)(p.block_table + (int64_t)r * p.max_pages);
    const int64_t v_plane = (int64_t)p.Hkv * kPS * kD; // K slab -> V slab inside a page
    const int64_t row_pitch = (int64_t)p.Hkv * kD;     // elements between rows of k_new

    // Full tiles (no row to clamp) take a shorter address path: a scalar base per page, or per
    // load step of the suffix, plus a per-lane byte offset that never changes.
    typedef const __attribute__((address_space(1))) char *gptr;
    const uint32_t row_bytes = (uint32_t)row_pitch * 2u;
    // Direct loads put lane i's 16 bytes into slot i of the wavefront's 1 KiB of LDS (4 rows of
    // 16 slots), so the swizzle is applied on the source side: slot s of row r holds chunk
    // s ^ (r & 15) of a K row and chunk s ^ ((r & 3) << 2) of a V row.
    const int ck = ld_chunk ^ (ld_row & 15);
    const int cv = ld_chunk ^ ((ld_row & 3) << 2);
    const uint32_t pg_lane_k = (uint32_t)(((ld_row & 15) * kD + ck * 8) * 2); // inside a page's K slab
    const uint32_t pg_lane_v = (uint32_t)(((ld_row & 15) * kD + cv * 8) * 2) + (uint32_t)(v_plane * 2);
    const uint32_t sfx_lane_k = (uint32_t)ld_row * row_bytes + (uint32_t)ck * 16u;
    const uint32_t sfx_lane_v = (uint32_t)ld_row * row_bytes + (uint32_t)cv * 16u;
    // Four direct loads of 16 bytes per lane: K and V rows ld_row and ld_row + 32 of buffer buf.
    // M0 carries the LDS address of the wavefront's 1 KiB.  The loads are written as assembly
    // because the compiler, for the builtin, waits for every direct load in flight before the
    // next LDS read of the wavefront, whichever buffer that read goes to; here the only reader
    // of the loaded buffer is two barriers away, and dma_wait() in front of each barrier is the
    // wait that is needed.  The compiler's own counts stay conservative: it does not see these
    // loads, loads complete in order, so its waits can only cover more than it meant.
    const uint32_t lds_k_wave = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds_k + wave * (4 * kPitchK);
    const uint32_t lds_v_wave = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds_v + wave * (4 * kPitchV);
    auto dma_tile = [&](gptr k0, gptr v0, gptr k1, gptr v1, int kbuf, int vbuf) {
        const uint32_t dk0 = __builtin_amdgcn_readfirstlane(lds_k_wave + kbuf * kTileBytesK);
        const uint32_t dv0 = __builtin_amdgcn_readfirstlane(lds_v_wave + vbuf * kTileBytesV);
        const uint32_t dk1 = dk0 + kLoadRows * kPitchK, dv1 = dv0 + kLoadRows * kPitchV;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %4, off\n\t"
                     "s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %5, off\n\t"
                     "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %6, off\n\t"
                     "s_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %7, off"
                     :
                     : "s"(dk0), "s"(dv0), "s"(dk1), "s"(dv1), "v"(k0), "v"(v0), "v"(k1), "v"(v1)
                     : "memory"); // m0 is reserved: the compiler keeps nothing in it across statements
    };
    // all of this wavefront's direct loads have landed (the barrier that follows publishes them)
    auto dma_wait = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
    const uint64_t page_bytes = (uint64_t)p.Hkv * (2u * kPS * kD * 2u);
    const gptr pages_head = (gptr)p.kv_pages + (int64_t)kvh * (kPS * kD * 2);
    const gptr knew_head = (gptr)p.k_new + ((int64_t)cu * p.Hkv + kvh) * (kD * 2);
    const gptr vnew_head = (gptr)p.v_new + ((int64_t)cu * p.Hkv + kvh) * (kD * 2);
    auto load_tile = [&](int kt, int t) { // t: tile number inside the work item
        const int kbuf = t & 3, vbuf = t % kNumBufsV;
        if (kt < np_tiles && (kt + 1) * kBN <= P) {
            gptr kp[2], vp[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t page = (uint32_t)table[kt * (kBN / kPS) + 2 * i + (wave >> 2)];
                const gptr base = pages_head + (uint64_t)page * page_bytes;
                kp[i] = base + pg_lane_k;
                vp[i] = base + pg_lane_v;
            }
            dma_tile(kp[0], vp[0], kp[1], vp[1], kbuf, vbuf);
            return;
        }
        if (kt >= np_tiles && (kt - np_tiles + 1) * kBN <= E) {
            const int64_t tile_off = (int64_t)(kt - np_tiles) * kBN * row_bytes;
            const int64_t off1 = tile_off + (int64_t)kLoadRows * row_bytes;
            dma_tile(knew_head + tile_off + sfx_lane_k, vnew_head + tile_off + sfx_lane_v,
                     knew_head + off1 + sfx_lane_k, vnew_head + off1 + sfx_lane_v, kbuf, vbuf);
            return;
        }
        const uint16_t *ks[2];
        const uint16_t *vs[2];
        if (kt < np_tiles) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int tok0 = min(kt * kBN + i * kLoadRows + wave * 4, P - 1); // wave-uniform
                const int sub = min(ld_sub, P - 1 - tok0);
                const int64_t page = table[tok0 >> 4];
                const uint16_t *base = p.kv_pages + (page * 2 * p.Hkv + kvh) * (kPS * kD);
                ks[i] = base + ((((tok0 + sub) & 15) * kD) + ck * 8);
                vs[i] = base + ((((tok0 + sub) & 15) * kD) + cv * 8) + v_plane;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int srow0 = min((kt - np_tiles) * kBN + i * kLoadRows + wave * 4, E - 1);
                const int sub = min(ld_sub, E - 1 - srow0);
                const int64_t base = ((int64_t)(cu + srow0) * p.Hkv + kvh) * kD;
                const int off = sub * (int)row_pitch;
                ks[i] = p.k_new + base + off + ck * 8;
                vs[i] = p.v_new + base + off + cv * 8;
            }
        }
        dma_tile((gptr)ks[0], (gptr)vs[0], (gptr)ks[1], (gptr)vs[1], kbuf, vbuf);
    };

    // ---- per-lane LDS read offsets (bytes inside a tile buffer)
    // K, A operand of S^T: lane (j, h) reads 16 bytes of key row kb*32 + j at chunk 2 kk + h,
    // which the swizzle puts at slot (2 kk + h) ^ (j & 15): one offset per kk.
    int k_lane[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) k_lane[kk] = j * kPitchK + (((2 * kk + h) ^ (j & 15)) << 4);
    // V^T, A operand of O^T = V^T P^T, through the transposing read: within a group of 16
    // lanes, lane i supplies the address of 4 consecutive d of key row k0 + i / 4 and receives
    // V[k0 .. k0+3][d0 + i].  Here k0 = 4 h (+ 8 for the second read), d0 = 32 db + 16 (lane/16 % 2);
    // the swizzle exchanges the 64-byte column blocks: block db of row r sits at db ^ (r & 3).
    int v_lane[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
        v_lane[db] = (4 * h + ((lane & 15) >> 2)) * kPitchV + ((db ^ ((lane >> 2) & 3)) << 6) + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;

    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m_ref = -INFINITY; // reference maximum of the exponentials, log2 domain
    float l_run = 0.f;       // running sum over this half-wave's keys only
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

    typedef f32x16 STile[kNKB];     // scores: 32-key blocks x 32 query rows
    typedef bf16x8 PTile[2 * kNKB]; // probabilities: one B operand per 16 keys

    // S^T = K Q^T for the tile in K buffer kbuf.
    auto qk_tile = [&](int kbuf, STile &s) {
        const char *kb = lds_k + kbuf * kTileBytesK;
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int b = 0; b < kNKB; ++b) s[b] = zero;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
            for (int b = 0; b < kNKB; ++b) {
                const u32x4 a = *reinterpret_cast<const u32x4 *>(kb + k_lane[kk] + b * 32 * kPitchK);
                s[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), qf[kk], s[b], 0, 0, 0);
            }
        }
        // Issue order: kFragsAhead fragment reads first, then one read behind every MFMA, so
        // that an operand is requested kFragsAhead MFMAs before it is used (left alone, the
        // scheduler reads two fragments and waits for them at once).
        constexpr int kFragsAhead = 8;
        __builtin_amdgcn_sched_group_barrier(0x100, kFragsAhead, 0);
#pragma unroll
        for (int i = 0; i < 8 * kNKB - kFragsAhead; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, kFragsAhead, 0);
    };
    // O^T += V^T P^T for the tile in V buffer vbuf: 4 d blocks x steps of 16 keys.
    auto pv_tile = [&](int vbuf, const PTile &pb) {
        const char *vb = lds_v + vbuf * kTileBytesV;
#pragma unroll
        for (int ks = 0; ks < 2 * kNKB; ++ks) { // keys ks*16 .. ks*16+15
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const char *a = vb + v_lane[db] + ks * 16 * kPitchV;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(a));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(a + 8 * kPitchV));
                const s16x8 vv = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pb[ks], o[db], 0, 0, 0);
            }
        }
        // Same for the V fragments (two transposing reads each), five MFMAs ahead, with up to
        // four VALU instructions of the next tile's softmax (64 in all: 32 exponentials, 16
        // conversions, 16 row-sum steps) behind every MFMA where the caller has them in the same
        // block.
        constexpr int kFragsAhead = 5;
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * kFragsAhead, 0);
#pragma unroll
        for (int i = 0; i < 8 * kNKB; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i < 8 * kNKB - kFragsAhead) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x400, 4, 0);
        }
    };
    // Masks the keys of a boundary tile that the lane's row must not see.  Accumulator element
    // v of block b is key b*32 + 8*(v/4) + 4*h + v%4 of the tile.
    auto mask_tile = [&](int vis, STile &s) {
        const int vis_h = vis - 4 * h;
#pragma unroll
        for (int b = 0; b < kNKB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (b * 32 + 8 * (v >> 2) + (v & 3) >= vis_h) s[b][v] = -INFINITY;
    };
    // Exponentials of one tile against the reference m_use (log2 domain), one query row per
    // lane: bf16 probabilities in B-operand order (pb[2b + u] element e is accumulator element
    // 8u + e of block b); returns their sum over this lane's keys.  `plain` says that the
    // reference is 0 for every row of the wavefront: then there is nothing to subtract.
    auto exp_tile = [&](const STile &s, PTile &pb, float m_use, auto plain) -> float {
        constexpr bool kPlain = decltype(plain)::value;
        float psum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e += 2)
#pragma unroll
            for (int t = 0; t < 2 * kNKB; ++t) {
                f32x2 x;
                const float s0 = s[t >> 1][8 * (t & 1) + e], s1 = s[t >> 1][8 * (t & 1) + e + 1];
                x[0] = fast_exp2(kPlain ? s0 : s0 - m_use);
                x[1] = fast_exp2(kPlain ? s1 : s1 - m_use);
                const bf16x2 y = __builtin_convertvector(x, bf16x2);
                psum = __builtin_amdgcn_fdot2_f32_bf16(y, ones, psum, false);
                pb[t][e] = y[0];
                pb[t][e + 1] = y[1];
            }
        return psum;
    };
    auto row_max = [&](const STile &s) -> float {
        float mx = s[0][0];
#pragma unroll
        for (int i = 1; i + 1 < 16 * kNKB; i += 2) // pairs, so that three-input maxima can be used
            mx = fmaxf(fmaxf(mx, s[i >> 4][i & 15]), s[(i + 1) >> 4][(i + 1) & 15]);
        mx = fmaxf(mx, s[kNKB - 1][15]);
        return halfwave_max(mx);
    };
    auto rescale_o = [&](float alpha) {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
    };

    // ---- main loop, one barrier per two key tiles.  Iteration `it`:
    //     request tile it+2: global memory -> K buffer (it+2) % 4, V buffer (it+2) % 5, asynchronously
    //     S = K(it) Q^T                                            (MFMA)
    //     p = exp2(S - m_ref) next to O += V(it-1)^T P(it-1)^T     (VALU next to MFMA)
    //     if `it` is even: wait for the requested tiles, barrier
    // (S already carries softmax_scale * log2(e), see the Q fragments.)  The exponentials are
    // taken against the running reference m_ref WITHOUT first reducing the row maximum of the
    // tile.  Only when some row of the wavefront has no reference yet, or its sum shows that the
    // reference is stale by a factor 2^80 or more, is the tile redone the classic way (row
    // maximum, new reference, rescale of O and l).  Any reference gives the same result after
    // the final division as long as nothing overflows or vanishes: a row maximum inside
    // [-kSnap, kSnap] takes the reference 0 (exponentials between 2^-64 and 2^64 at the top of
    // the row, nothing to subtract), and below the trigger the sums stay under 2^80 times the
    // number of keys, which fp32 holds up to 2^47 keys of magnitude 1.
    load_tile(kt_begin, 0);
    if (n_it > 1) load_tile(kt_begin + 1, 1);
    dma_wait();
    __syncthreads();

    bool have_prev = false; // the previous tile's probabilities still wait for their P V
    constexpr float kStale = 1.2089258196146292e24f; // 2^80
    constexpr float kSnap = 64.f; // a row whose maximum lies in [-64, 64] takes the reference 0

    // Classic online-softmax step: row maximum, new reference, rescale of O and l.
    auto redo_tile = [&](const STile &s, PTile &pb) -> float {
        float m_new = fmaxf(m_ref, row_max(s));
        if (fabsf(m_new) <= kSnap) m_new = 0.f;
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2(m_ref - m_use);
        rescale_o(alpha);
        l_run *= alpha;
        m_ref = m_new;
        return exp_tile(s, pb, m_use, std::false_type{});
    };
    // first key of tile kt in its own numbering (prefix tokens or suffix rows)
    auto tile_key0 = [&](int kt) { return kt >= np_tiles ? (kt - np_tiles) * kBN : kt * kBN; };
    auto masked_qk = [&](int kt, int buf, STile &s) {
        const bool suffix = kt >= np_tiles;
        const int key0 = tile_key0(kt);
        qk_tile(buf, s);
        const bool need_mask = suffix ? (key0 + kBN - 1 > wave_row0) : (key0 + kBN > P);
        if (need_mask) mask_tile(suffix ? (row_i - key0 + 1) : (P - key0), s);
    };
    // a suffix tile entirely above this wavefront's rows shows it nothing, and neither does
    // any later tile; a wavefront whose 32 rows all lie past the end of the request (short
    // extends, decode) computes nothing at all and only takes part in the cooperative loads
    const bool no_rows = wave_row0 >= E;
    auto skipped = [&](int kt) { return no_rows || (kt >= np_tiles && tile_key0(kt) > wave_row0 + 31); };

    PTile pb_a, pb_b; // probabilities of the previous / the current tile

    // iteration 0: no previous tile yet, and no reference: classic step
    {
        const bool prefetch = 2 < n_it;
        if (prefetch) load_tile(kt_begin + 2, 2);
        if (!skipped(kt_begin)) {
            STile s;
            masked_qk(kt_begin, 0, s);
            l_run += redo_tile(s, pb_a);
            have_prev = true;
        }
        dma_wait();
        __syncthreads();
    }
    // The barrier comes after every second tile (after the even ones): a function of the tile
    // number alone, so every wavefront meets the same barriers whichever loop it is in.
    auto pair_barrier = [&](int it) {
        if (!(it & 1)) {
            dma_wait();
            __syncthreads();
        }
    };
    // One full step; only called for tiles this wavefront does not skip (so the previous tile
    // was not skipped either and its probabilities are pending).
    auto tile_step = [&](int it, PTile &pb_cur, PTile &pb_prev) {
        const int buf = it & 3;
        const int kt = kt_begin + it;
        const bool prefetch = it + 2 < n_it;
        if (prefetch) load_tile(kt + 2, it + 2);
        STile s;
        masked_qk(kt, buf, s);
        // one basic block: the exponentials (VALU) interleave with P V (MFMA)
        float psum = exp_tile(s, pb_cur, (m_ref == -INFINITY) ? 0.f : m_ref, std::false_type{});
        pv_tile((it - 1) % kNumBufsV, pb_prev);
        if (__builtin_amdgcn_ballot_w64(!(psum < kStale) || m_ref == -INFINITY) != 0)
            psum = redo_tile(s, pb_cur);
        l_run += psum;
        pair_barrier(it);
    };
    int it = 1;
    if (have_prev) {
        // Steady state: while tile kt needs no mask for this wavefront and tile kt + 2 is a
        // full tile (inside the prefix, or suffix rows below the diagonal), the step has no
        // case distinctions, and the block-table entries of a tile are fetched one iteration
        // before its loads are issued (the general step spends ~500 of ~4200 cycles per tile
        // between the barrier and its first MFMA on tile kinds, table lookups and addresses,
        // with the matrix pipe idle).
        int fast_end;
        if (P % kBN == 0) {
            const int last_unmasked = np_tiles + (wave_row0 >= kBN - 1 ? (wave_row0 - (kBN - 1)) / kBN : -1);
            const int last_full = np_tiles + E / kBN - 1;
            fast_end = min(min(last_unmasked + 1, last_full - 1), kt_end - 2) - kt_begin;
        } else {
            fast_end = min(n_it - 2, P / kBN - 2 - kt_begin);
        }
        if (it < fast_end) {
            const int tsel = wave >> 2;
            const int last_entry = (P + E + kPS - 1) / kPS - 1; // last page of the request: nothing beyond it is read
            auto entry = [&](int kt, int i) {
                return (uint32_t)table[min(kt * (kBN / kPS) + 2 * i + tsel, last_entry)];
            };
            uint32_t pg0 = entry(kt_begin + it + 2, 0), pg1 = entry(kt_begin + it + 2, 1);
            int vprev = (it - 1) % kNumBufsV; // V buffer of tile it - 1
            auto vnext = [](int v, int n) { v += n; return v >= kNumBufsV ? v - kNumBufsV : v; };
            // while every row of the wavefront has the reference 0 (the usual case, see kSnap);
            // otherwise the general step below takes over
            for (; it < fast_end && __builtin_amdgcn_ballot_w64(m_ref != 0.f) == 0; ++it) {
                const int buf = it & 3;
                const int kt2 = kt_begin + it + 2;
                gptr k0, v0, k1, v1;
                if (kt2 < np_tiles) {
                    const gptr b0 = pages_head + (uint64_t)pg0 * page_bytes;
                    const gptr b1 = pages_head + (uint64_t)pg1 * page_bytes;
                    k0 = b0 + pg_lane_k;
                    v0 = b0 + pg_lane_v;
                    k1 = b1 + pg_lane_k;
                    v1 = b1 + pg_lane_v;
                } else {
                    const int64_t off = (int64_t)(kt2 - np_tiles) * kBN * row_bytes;
                    k0 = knew_head + off + sfx_lane_k;
                    v0 = vnew_head + off + sfx_lane_v;
                    k1 = k0 + (int64_t)kLoadRows * row_bytes;
                    v1 = v0 + (int64_t)kLoadRows * row_bytes;
                }
                dma_tile(k0, v0, k1, v1, (buf + 2) & 3, vnext(vprev, 3));
                pg0 = entry(kt_begin + it + 3, 0);
                pg1 = entry(kt_begin + it + 3, 1);
                STile s;
                qk_tile(buf, s);
                float psum = exp_tile(s, pb_b, 0.f, std::true_type{});
                pv_tile(vprev, pb_a);
                if (__builtin_amdgcn_ballot_w64(!(psum < kStale) || m_ref == -INFINITY) != 0)
                    psum = redo_tile(s, pb_b);
                l_run += psum;
                pair_barrier(it);
                vprev = vnext(vprev, 1);
#pragma unroll
                for (int t = 0; t < 2 * kNKB; ++t) pb_a[t] = pb_b[t];
            }
        }
        // the general step: one call site, so that the accumulators stay in the same registers
        for (; it < n_it && !skipped(kt_begin + it); ++it) {
            tile_step(it, pb_b, pb_a);
#pragma unroll
            for (int t = 0; t < 2 * kNKB; ++t) pb_a[t] = pb_b[t];
        }
        // P V of the last tile this wavefront computed (tile it - 1)
        pv_tile((it - 1) % kNumBufsV, pb_a);
    }
    // remaining tiles are invisible to this wavefront: only take part in the cooperative loads
    for (; it < n_it; ++it) {
        const bool prefetch = it + 2 < n_it;
        if (prefetch) {
            load_tile(kt_begin + it + 2, it + 2);
        }
        pair_barrier(it);
    }

    // ---- epilogue.  o[db][v] is O^T[d = db*32 + 8*(v/4) + 4*h + v%4][row j]
    const float l_tot = halfwave_sum(l_run);
    if (!row_valid) return;
    if (kSplit) {
        const int64_t prow = ((int64_t)split * p.T + out_row) * p.Hq + head;
        float *po = p.part_o + prow * kD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                f32x4 x = {o[db][4 * gq], o[db][4 * gq + 1], o[db][4 * gq + 2], o[db][4 * gq + 3]};
                *reinterpret_cast<f32x4 *>(po + db * 32 + 8 * gq + 4 * h) = x;
            }
        if (h == 0) {
            p.part_ml[prow * 2] = m_ref;
            p.part_ml[prow * 2 + 1] = l_tot;
        }
    } else {
        const float inv = 1.f / l_tot;
        uint16_t *po = p.out + (out_row * p.Hq + head) * kD;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                bf16x4 x;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = (__bf16)(o[db][4 * gq + e] * inv);
                *reinterpret_cast<bf16x4 *>(po + db * 32 + 8 * gq + 4 * h) = x;
            }
    }
}

// out[row, head, :] = sum_s w_s O_s / sum_s w_s l_s with w_s = 2^(m_s - max_s m_s).
// Entries with l_s = 0 (empty splits) are skipped.  Two forms, chosen by the number of splits; in
// both every sum runs in a fixed order, so the result is reproducible.
//
// Many splits: one workgroup per (row, head).  kMergeGroups groups of 32 threads take the splits
// s = g, g + kMergeGroups, ... (at most kMergePerGroup each; 4 consecutive d per thread), then the
// partial sums of the groups are added in group order.
constexpr int kMergeGroups = 32;
constexpr int kMergePerGroup = 8; // splits per group: up to 256 partial results in all
constexpr int kMergeFewSplits = 8; // up to this many splits the second form is used
__global__ __launch_bounds__(32 * kMergeGroups) void merge_splits_kernel(const float *__restrict__ part_o,
                                                                          const float *__restrict__ part_ml,
                                                                          uint16_t *__restrict__ out,
                                                                          int64_t n_rh, int nsplit)
{
    __shared__ float s_max[kMergeGroups];
    __shared__ float s_den[kMergeGroups];
    __shared__ f32x4 s_acc[kMergeGroups][32];
    const int64_t rh = blockIdx.x;
    const int g = threadIdx.x >> 5, t = threadIdx.x & 31;
    const int d4 = t * 4;
    // all loads of the group first (one round of memory latency), then the arithmetic
    float ms[kMergePerGroup], ls[kMergePerGroup];
    f32x4 x[kMergePerGroup];
#pragma unroll
    for (int i = 0; i < kMergePerGroup; ++i) {
        const int s = g + i * kMergeGroups;
        const bool on = s < nsplit;
        const f32x2 ml = on ? *reinterpret_cast<const f32x2 *>(part_ml + ((int64_t)s * n_rh + rh) * 2) : f32x2{0.f, 0.f};
        ms[i] = ml[0];
        ls[i] = ml[1];
        x[i] = on ? *reinterpret_cast<const f32x4 *>(part_o + ((int64_t)s * n_rh + rh) * kD + d4) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // maximum over all splits: inside the group every thread holds the same values; across groups
    // through LDS
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < kMergePerGroup; ++i)
        if (ls[i] > 0.f) m = fmaxf(m, ms[i]);
    if (t == 0) s_max[g] = m;
    __syncthreads();
    float m_star = s_max[0];
#pragma unroll
    for (int i = 1; i < kMergeGroups; ++i) m_star = fmaxf(m_star, s_max[i]);

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float denom = 0.f;
#pragma unroll
    for (int i = 0; i < kMergePerGroup; ++i)
        if (ls[i] > 0.f) {
            const float w = fast_exp2(ms[i] - m_star);
            acc += x[i] * w;
            denom += ls[i] * w;
        }
    s_acc[g][t] = acc;
    if (t == 0) s_den[g] = denom;
    __syncthreads();
    if (g != 0) return;
#pragma unroll
    for (int i = 1; i < kMergeGroups; ++i) {
        acc += s_acc[i][t];
        denom += s_den[i];
    }
    const float inv = denom > 0.f ? 1.f / denom : 0.f;
    bf16x4 y;
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = (__bf16)(acc[e] * inv);
    *reinterpret_cast<bf16x4 *>(out + rh * kD + d4) = y;
}

// Few splits: a group of 32 threads per (row, head), eight of them per workgroup, each walking
// over its splits in order with all loads of a pass in flight together.
template <int kSplits>
__global__ __launch_bounds__(256) void merge_few_splits_kernel(const float *__restrict__ part_o,
                                                               const float *__restrict__ part_ml,
                                                               uint16_t *__restrict__ out, int64_t n_rh, int nsplit)
{
    const int64_t rh = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);
    if (rh >= n_rh) return;
    const int d4 = (threadIdx.x & 31) * 4;
    float ms[kSplits], ls[kSplits];
    f32x4 x[kSplits];
#pragma unroll
    for (int s = 0; s < kSplits; ++s) {
        const bool on = s < nsplit;
        const f32x2 ml = on ? *reinterpret_cast<const f32x2 *>(part_ml + ((int64_t)s * n_rh + rh) * 2) : f32x2{0.f, 0.f};
        ms[s] = ml[0];
        ls[s] = ml[1];
        x[s] = on ? *reinterpret_cast<const f32x4 *>(part_o + ((int64_t)s * n_rh + rh) * kD + d4) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    float m_star = -INFINITY;
#pragma unroll
    for (int s = 0; s < kSplits; ++s)
        if (ls[s] > 0.f) m_star = fmaxf(m_star, ms[s]);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float denom = 0.f;
#pragma unroll
    for (int s = 0; s < kSplits; ++s)
        if (ls[s] > 0.f) {
            const float w = fast_exp2(ms[s] - m_star);
            acc += x[s] * w;
            denom += ls[s] * w;
        }
    const float inv = denom > 0.f ? 1.f / denom : 0.f;
    bf16x4 y;
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = (__bf16)(acc[e] * inv);
    *reinterpret_cast<bf16x4 *>(out + rh * kD + d4) = y;
}

// ---- decode-shaped calls ------------------------------------------------------------------
// When every request brings so few new tokens that all its rows for one KV head (G heads x E_r
// tokens) fit a few 32-column MFMA tiles, the call is bound by reading the cached K/V once,
// and the row-tiled kernel above wastes its wavefronts (most hold no valid row) and keeps too
// little in flight.  This kernel turns the work around: a wavefront is the unit, owns 32 rows
// of one (request, KV head) and a contiguous chunk of the keys, and runs alone - no barrier, no
// shared tile.  Per block of 32 keys it loads the K and V rows with fully coalesced 16-byte
// loads (one instruction = four whole rows), stages them in registers while the previous block
// is computed, and passes them through a private LDS area from which the MFMA operands are read
// (K rows as they are, V rows transposed).  Every wavefront writes an unnormalised partial
// (m, l, O) and merge_splits_kernel combines them, exactly as for split-K.  Prefix and suffix
// keys form one sequence of N = P + E keys; blocks inside the prefix take their two pages from
// the block table with scalar loads, the last blocks resolve every row on its own.
constexpr int kDecRows = 32;            // (head, token) rows per wavefront
constexpr int kDecMaxRowBlocks = 2;     // row blocks per (request, KV head): G x E_r <= 64 (beyond, the row-tiled kernel is faster)
constexpr int kDecWaves = 4;            // wavefronts per workgroup (independent of each other)
// LDS bytes per K row / V row: 256 + padding.  16 consecutive K rows at the same column fall into
// 16 different 16-byte bank groups, the four consecutive V rows of a transposing read into four
// different 64-byte bank groups, and every read address is a per-lane base plus an immediate.
constexpr int kDecPitchK = 272;
constexpr int kDecPitchV = 320;
constexpr int kDecLdsK = 32 * kDecPitchK;
constexpr int kDecLdsPerWave = kDecLdsK + 32 * kDecPitchV;
constexpr int kDecMaxChunks = 256;      // key chunks (= partial results) per (request, KV head)
static_assert(kDecMaxChunks <= kMergeGroups * kMergePerGroup && kMaxSplits <= kMergeGroups * kMergePerGroup,
              "the merge kernel holds all partial results of a row in registers");

struct DecBlock { // one block of 32 keys as loaded: piece i is row (lane / 16) + 4 i, chunk lane % 16
    u32x4 k[8];
    u32x4 v[8];
};

__global__ __launch_bounds__(kDecWaves * 64, 2) void decode_attn_kernel(const AttnParams p)
{
    __shared__ __attribute__((aligned(16))) char lds[kDecWaves * kDecLdsPerWave];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int j = lane & 31; // (head, token) row of the accumulators; key row of the K operand
    const int h = lane >> 5;
    char *const lds_k = lds + wave * kDecLdsPerWave;
    char *const lds_v = lds_k + kDecLdsK;

    // work unit: row block fastest (neighbouring wavefronts then read the same keys), then key
    // chunk, KV head, request
    const int64_t unit = (int64_t)blockIdx.x * kDecWaves + wave;
    const int rb = (int)(unit % p.dec_row_blocks);
    const int64_t uc = unit / p.dec_row_blocks;
    const int chunk = (int)(uc % p.nsplit);
    const int64_t rk = uc / p.nsplit;
    const int kvh = (int)(rk % p.Hkv);
    const int r = (int)(rk / p.Hkv);
    if (r >= p.batch) return;
    const int E = p.extend_lens[r];
    if (E <= 0) return;
    const int P = p.prefix_lens[r];
    // packed row of the request's first token: sum of the earlier extend lengths, 64 per step
    int cu = 0;
    for (int base = 0; base < r; base += 64) cu += base + lane < r ? p.extend_lens[base + lane] : 0;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) cu += __shfl_xor(cu, off, 64);
    cu = __builtin_amdgcn_readfirstlane(cu);
    const int N = P + E;
    const int nblk = (N + 31) >> 5;
    const int per = (nblk + p.nsplit - 1) / p.nsplit;
    const int b0 = chunk * per;
    const int b1 = min(nblk, b0 + per);

    // row 32 rb + j of the (request, KV head) is token e of head hg of the group; rows beyond
    // G E are padding
    if (rb * kDecRows >= p.G * E) return;
    const int row = rb * kDecRows + j;
    const bool row_valid = row < p.G * E;
    const int hg = row_valid ? row / E : 0;
    const int e = row_valid ? row - hg * E : 0;
    const int head = kvh * p.G + hg;
    const int64_t out_row = cu + e;
    const int64_t prow = ((int64_t)chunk * p.T + out_row) * p.Hq + head;
    if (b0 >= b1) { // nothing to do for this chunk: the merge skips entries whose sum is zero
        if (row_valid && h == 0) {
            p.part_ml[prow * 2] = -INFINITY;
            p.part_ml[prow * 2 + 1] = 0.f;
        }
        return;
    }

    // Q fragments, B operand of S^T = K Q^T: lane (row j, h) holds q[row][16 kk + 8 h .. + 8)
    u32x4 qf[8];
    {
        const uint16_t *qp = p.q + (out_row * p.Hq + head) * kD + 8 * h;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) qf[kk] = *(const __attribute__((address_space(1))) u32x4 *)(qp + 16 * kk);
    }

    // loads: lane covers rows ld_sub + 4 i (i = 0..7) of the block, 16-byte chunk ld_chunk
    const int ld_sub = lane >> 4, ld_chunk = lane & 15;
    const __attribute__((address_space(4))) int32_t *table =
        (const __attribute__((address_space(4))) int32_t *)(p.block_table + (int64_t)r * p.max_pages);
    const int64_t v_plane = (int64_t)p.Hkv * kPS * kD;
    const int64_t page_stride = 2 * v_plane;
    const uint16_t *pages_head = p.kv_pages + (int64_t)kvh * (kPS * kD) + ld_chunk * 8;
    auto load_block = [&](int b, DecBlock &blk) {
        if (b * 32 + 32 <= P) {
            // inside the prefix: rows 0..15 in page 2 b, rows 16..31 in page 2 b + 1
            const int64_t pg[2] = {table[2 * b], table[2 * b + 1]};
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint16_t *krow = pages_head + pg[i >> 2] * page_stride + ((ld_sub + 4 * i) & 15) * kD;
                blk.k[i] = *(const __attribute__((address_space(1))) u32x4 *)(krow);
                blk.v[i] = *(const __attribute__((address_space(1))) u32x4 *)(krow + v_plane);
            }
        } else {
            // last blocks: every row resolves its own key (clamped to the last one; masked below)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int key = min(b * 32 + ld_sub + 4 * i, N - 1);
                const uint16_t *krow, *vrow;
                if (key < P) {
                    krow = pages_head + (int64_t)p.block_table[(int64_t)r * p.max_pages + (key >> 4)] * page_stride +
                           (key & 15) * kD;
                    vrow = krow + v_plane;
                } else {
                    const int64_t off = ((int64_t)(cu + key - P) * p.Hkv + kvh) * kD + ld_chunk * 8;
                    krow = p.k_new + off;
                    vrow = p.v_new + off;
                }
                blk.k[i] = *(const __attribute__((address_space(1))) u32x4 *)(krow);
                blk.v[i] = *(const __attribute__((address_space(1))) u32x4 *)(vrow);
            }
        }
    };
    const int st_k = ld_sub * kDecPitchK + ld_chunk * 16;
    const int st_v = ld_sub * kDecPitchV + ld_chunk * 16;
    auto store_block = [&](const DecBlock &blk) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            *reinterpret_cast<u32x4 *>(lds_k + st_k + 4 * i * kDecPitchK) = blk.k[i];
            *reinterpret_cast<u32x4 *>(lds_v + st_v + 4 * i * kDecPitchV) = blk.v[i];
        }
    };
    // operand reads, as in the kernel above
    const int k_lane = j * kDecPitchK + h * 16;
    const int v_lane = (4 * h + ((lane & 15) >> 2)) * kDecPitchV + ((lane >> 4) & 1) * 32 + (lane & 3) * 8;

    f32x16 o[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f; // log2 domain; sum over this half-wave's keys
    const float c = p.scale_log2;
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};

    DecBlock blk;
    load_block(b0, blk);
    for (int b = b0; b < b1; ++b) {
        // block b: registers -> private LDS (one wavefront's LDS operations are served in order,
        // so these writes come after the reads of block b - 1), then block b + 1 into flight
        store_block(blk);
        if (b + 1 < b1) load_block(b + 1, blk);
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const u32x4 a = *reinterpret_cast<const u32x4 *>(lds_k + k_lane + kk * 32);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                         __builtin_bit_cast(bf16x8, qf[kk]), s, 0, 0, 0);
        }
        // accumulator element v is key 32 b + 8 (v / 4) + 4 h + v % 4; row j sees keys <= P + e
        if (b * 32 + 31 > P) {
            const int vis = P + e - b * 32 - 4 * h; // visible: 8 (v / 4) + v % 4 <= vis
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (8 * (v >> 2) + (v & 3) > vis) s[v] = -INFINITY;
        }
        float mx = s[0];
#pragma unroll
        for (int v = 1; v + 1 < 16; v += 2) mx = fmaxf(fmaxf(mx, s[v]), s[v + 1]);
        mx = halfwave_max(fmaxf(mx, s[15]));
        const float m_new = fmaxf(m_run, mx * c);
        const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = fast_exp2(m_run - m_use);
        u32x4 pb[2];
        float psum = 0.f;
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                f32x2 x;
                x[0] = fast_exp2(fmaf(s[8 * u + 2 * w], c, -m_use));
                x[1] = fast_exp2(fmaf(s[8 * u + 2 * w + 1], c, -m_use));
                const bf16x2 y = __builtin_convertvector(x, bf16x2);
                psum = __builtin_amdgcn_fdot2_f32_bf16(y, ones, psum, false);
                pb[u][w] = __builtin_bit_cast(unsigned, y);
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
        }
        // O^T += V^T P^T: 2 steps of 16 keys x 4 blocks of 32 d
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const char *a = lds_v + v_lane + db * 64 + ks * 16 * kDecPitchV;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(a));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(a + 8 * kDecPitchV));
                const s16x8 vv = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv),
                                                                 __builtin_bit_cast(bf16x8, pb[ks]), o[db], 0, 0, 0);
            }
    }

    // partial result of this chunk; o[db][v] is O^T[d = db*32 + 8*(v/4) + 4*h + v%4][row j]
    const float l_tot = halfwave_sum(l_run);
    if (!row_valid) return;
    float *po = p.part_o + prow * kD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            f32x4 x = {o[db][4 * gq], o[db][4 * gq + 1], o[db][4 * gq + 2], o[db][4 * gq + 3]};
            *reinterpret_cast<f32x4 *>(po + db * 32 + 8 * gq + 4 * h) = x;
        }
    if (h == 0) {
        p.part_ml[prow * 2] = m_run;
        p.part_ml[prow * 2 + 1] = l_tot;
    }
}

// One workgroup copies 16 consecutive packed rows.  Its first wavefront finds the request, the
// page and the slot of every row, 64 requests at a time (a prefix sum of extend_lens across the
// lanes; a sequential scan costs one dependent load per request, which made a 32-row call take
// 30 us); then thread (row, 16-byte chunk) copies the row's K and V for every KV head.
constexpr int kWriteRows = 16;
__global__ __launch_bounds__(256) void write_kv_kernel(const uint16_t *__restrict__ k_new,
                                                       const uint16_t *__restrict__ v_new,
                                                       uint16_t *__restrict__ kv_pages,
                                                       const int32_t *__restrict__ block_table,
                                                       const int32_t *__restrict__ prefix_lens,
                                                       const int32_t *__restrict__ extend_lens,
                                                       int batch, int Hkv, int max_pages, int T)
{
    __shared__ int64_t s_page[kWriteRows]; // physical page of the row's token, -1: no such row
    __shared__ int s_slot[kWriteRows];     // its slot inside the page
    const int row0 = blockIdx.x * kWriteRows;
    const int lane = threadIdx.x & 63;
    if (threadIdx.x < 64) {
        int req = -1, off = 0; // lane i < 16: owner of row row0 + i and the row's index inside it
        int cu = 0;            // rows of the requests before `base`
        for (int base = 0; base < batch; base += 64) {
            const int rr = base + lane;
            const int e = rr < batch ? extend_lens[rr] : 0;
            const int incl = wave_inclusive_scan(e, lane);
            const int total = __builtin_amdgcn_readlane(incl, 63);
#pragma unroll
            for (int i = 0; i < kWriteRows; ++i) {
                const int t = row0 + i - cu; // the row's index among the rows of this group of requests
                if (t >= 0 && t < total) {
                    const int first = __builtin_ctzll(__builtin_amdgcn_ballot_w64(incl > t));
                    const int before = __builtin_amdgcn_readlane(incl - e, first);
                    if (lane == i) {
                        req = base + first;
                        off = t - before;
                    }
                }
            }
            if (row0 + kWriteRows - 1 - cu < total) break;
            cu += total;
        }
        if (lane < kWriteRows) {
            int64_t page = -1;
            int slot = 0;
            if (req >= 0 && row0 + lane < T) {
                const int tok = prefix_lens[req] + off;
                page = block_table[(int64_t)req * max_pages + (tok >> 4)];
                slot = tok & 15;
            }
            s_page[lane] = page;
            s_slot[lane] = slot;
        }
    }
    __syncthreads();
    const int lr = threadIdx.x >> 4; // row of the block
    const int ch = threadIdx.x & 15; // 16-byte chunk of a 256-byte head row
    const int64_t page = s_page[lr];
    if (page < 0) return;
    const int64_t row = row0 + lr;
    const uint16_t *ksrc = k_new + row * Hkv * kD + ch * 8;
    const uint16_t *vsrc = v_new + row * Hkv * kD + ch * 8;
    uint16_t *kdst = kv_pages + ((page * 2 * Hkv) * kPS + s_slot[lr]) * (int64_t)kD + ch * 8;
    uint16_t *vdst = kdst + (int64_t)Hkv * kPS * kD;
    const int64_t head_pitch = (int64_t)kPS * kD; // one KV head's slab inside a page
    int g = 0;
    for (; g + 2 <= Hkv; g += 2) { // four independent copies in flight
        const uint4 k0 = *reinterpret_cast<const uint4 *>(ksrc + (int64_t)g * kD);
        const uint4 k1 = *reinterpret_cast<const uint4 *>(ksrc + (int64_t)(g + 1) * kD);
        const uint4 v0 = *reinterpret_cast<const uint4 *>(vsrc + (int64_t)g * kD);
        const uint4 v1 = *reinterpret_cast<const uint4 *>(vsrc + (int64_t)(g + 1) * kD);
        *reinterpret_cast<uint4 *>(kdst + g * head_pitch) = k0;
        *reinterpret_cast<uint4 *>(kdst + (g + 1) * head_pitch) = k1;
        *reinterpret_cast<uint4 *>(vdst + g * head_pitch) = v0;
        *reinterpret_cast<uint4 *>(vdst + (g + 1) * head_pitch) = v1;
    }
    for (; g < Hkv; ++g) {
        *reinterpret_cast<uint4 *>(kdst + g * head_pitch) = *reinterpret_cast<const uint4 *>(ksrc + (int64_t)g * kD);
        *reinterpret_cast<uint4 *>(vdst + g * head_pitch) = *reinterpret_cast<const uint4 *>(vsrc + (int64_t)g * kD);
    }
}


// ---- optional check of the device-side tables ------------------------------------------------
// The attention and append kernels trust block_table and the device copies of the lengths.  This
// kernel reads them without following any page id: thread (request r, slot i) looks at
// block_table[r][i] for the slots the request uses, i < ceil((P_r + E_r) / 16), with P_r and E_r
// taken from the device arrays, and records the first offence (smallest code of request and slot)
// in one 64-bit word.
constexpr int kCheckThreads = 256;
enum : uint32_t { kCheckOk = 0u, kCheckBadLength = 1u, kCheckBadPage = 2u };
__global__ __launch_bounds__(kCheckThreads) void check_tables_kernel(const int32_t *__restrict__ block_table,
                                                                     const int32_t *__restrict__ prefix_lens,
                                                                     const int32_t *__restrict__ extend_lens,
                                                                     int batch, int max_pages, int num_pages,
                                                                     unsigned long long *__restrict__ first_bad)
{
    const int r = blockIdx.y;
    if (r >= batch) return;
    const int64_t P = prefix_lens[r], E = extend_lens[r];
    const int64_t used = (P + E + kPS - 1) / kPS;
    // key of an offence: kind in the top bits so that a bad length outranks a bad page, then the
    // request, then the slot; the smallest key wins
    auto report = [&](uint32_t kind, int slot) {
        const unsigned long long key = ((unsigned long long)(kind == kCheckBadLength ? 0u : 1u) << 62) |
                                       ((unsigned long long)(uint32_t)r << 31) | (unsigned long long)(uint32_t)slot;
        atomicMin(first_bad, key);
    };
    if (P < 0 || E < 0 || used > max_pages) {
        if (blockIdx.x == 0 && threadIdx.x == 0) report(kCheckBadLength, 0);
        return;
    }
    for (int64_t i = (int64_t)blockIdx.x * kCheckThreads + threadIdx.x; i < used; i += (int64_t)gridDim.x * kCheckThreads) {
        const int32_t page = block_table[(int64_t)r * max_pages + i];
        if (page < 0 || page >= num_pages) report(kCheckBadPage, (int)i);
    }
}

// Scratch of the check above and of the entry point that takes no workspace: file-scope device
// arrays, so that no call allocates.  In host code the arrays' names are stand-ins, not device
// addresses; the per-device address comes from hipGetSymbolAddress (device_scratch below).
__device__ __align__(256) unsigned long long g_check_report[32];

// ------------------------------------------------------------------ host side
struct Plan {
    int64_t q_tiles;   // work units per KV head: row tiles x head groups, summed over requests
    int32_t max_key_tiles;
    int32_t nsplit;
    bool decode;       // few rows per (request, KV head): decode_attn_kernel
    int32_t row_blocks; // ... in this many blocks of 32 rows
};

// Compute units of the device the first caller runs on (every device this library is built
// for has the same count); read once, any number of host threads may race to be that caller.
int num_cus()
{
    static std::atomic<int> cached{0};
    int n = cached.load(std::memory_order_relaxed);
    if (n == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached.store(n, std::memory_order_relaxed);
    }
    return n;
}

// The attention kernel uses more LDS than the default per-workgroup limit; raise it once.
bool allow_large_lds()
{
    static std::once_flag once;
    static bool ok = false;
    std::call_once(once, [] {
        const hipError_t a = hipFuncSetAttribute(reinterpret_cast<const void *>(&extend_attn_kernel<false>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        const hipError_t b = hipFuncSetAttribute(reinterpret_cast<const void *>(&extend_attn_kernel<true>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
        ok = a == hipSuccess && b == hipSuccess;
    });
    return ok;
}

int validate(const cp_shape *s)
{
    if (!s) return CP_ERR_NULL;
    if (!s->h_prefix_lens || !s->h_extend_lens) return CP_ERR_NULL;
    if (s->batch < 1 || s->num_q_heads < 1 || s->num_kv_heads < 1) return CP_ERR_SHAPE;
    if (s->num_q_heads % s->num_kv_heads != 0) return CP_ERR_SHAPE;
    if (s->head_dim != kD || s->page_size != kPS) return CP_ERR_SHAPE;
    if (s->num_pages < 1 || s->max_pages_per_req < 1 || s->total_extend < 0) return CP_ERR_SHAPE;
    if (!(s->softmax_scale > 0.f) || !(s->softmax_scale < 3.0e38f)) return CP_ERR_SHAPE;
    if (s->num_splits < 0 || s->num_splits > kMaxSplits) return CP_ERR_SHAPE;
    int64_t sum = 0;
    for (int r = 0; r < s->batch; ++r) {
        const int64_t P = s->h_prefix_lens[r], E = s->h_extend_lens[r];
        if (P < 0 || E < 0) return CP_ERR_SHAPE;
        if ((P + E + kPS - 1) / kPS > s->max_pages_per_req) return CP_ERR_SHAPE;
        if (P + E > INT32_MAX - 2 * kBM) return CP_ERR_SHAPE;
        sum += E;
    }
    if (sum != s->total_extend) return CP_ERR_SHAPE;
    return CP_OK;
}

Plan make_plan(const cp_shape *s)
{
    Plan pl{0, 0, 1, false, 1};
    const int G = s->num_q_heads / s->num_kv_heads;
    int64_t max_e = 0, max_n = 0;
    for (int r = 0; r < s->batch; ++r) {
        if (s->h_extend_lens[r] == 0) continue;
        max_e = std::max<int64_t>(max_e, s->h_extend_lens[r]);
        max_n = std::max<int64_t>(max_n, (int64_t)s->h_prefix_lens[r] + s->h_extend_lens[r]);
    }
    if (s->num_splits == 0 && max_e > 0 && max_e * G <= kDecRows * kDecMaxRowBlocks) {
        // Decode-shaped: one wavefront per (request, KV head, 32 rows, key chunk).  Enough chunks
        // for 8 wavefronts per CU, at least 2 blocks of 32 keys each, a multiple of the workgroup
        // size.
        pl.row_blocks = (int32_t)((max_e * G + kDecRows - 1) / kDecRows);
        const int64_t pairs = (int64_t)s->batch * s->num_kv_heads * pl.row_blocks;
        int64_t ns = (8LL * num_cus() + pairs - 1) / pairs;
        const int64_t cap = ((max_n + 31) / 32 + 1) / 2;
        if (ns > cap) ns = cap;
        ns = (ns + kDecWaves - 1) / kDecWaves * kDecWaves;
        if (ns > kDecMaxChunks) ns = kDecMaxChunks;
        if (ns < kDecWaves) ns = kDecWaves;
        pl.nsplit = (int32_t)ns;
        pl.decode = true;
        return pl;
    }
    for (int r = 0; r < s->batch; ++r) {
        const int64_t P = s->h_prefix_lens[r], E = s->h_extend_lens[r];
        if (E == 0) continue;
        const int pack = heads_per_tile((int)E, s->num_q_heads / s->num_kv_heads);
        pl.q_tiles += units_of_request((int)E, s->num_q_heads / s->num_kv_heads, pack);
        const int64_t kt = (P + kBN - 1) / kBN + (E + kBN - 1) / kBN;
        if (kt > pl.max_key_tiles) pl.max_key_tiles = (int32_t)kt;
    }
    if (s->num_splits >= 1) {
        pl.nsplit = s->num_splits;
    } else {
        // Split the keys only when the unsplit grid cannot give every CU two workgroups, and
        // never into pieces shorter than 8 key tiles.
        const int64_t items = pl.q_tiles * s->num_kv_heads;
        const int64_t want = 2LL * num_cus();
        int64_t ns = 1;
        if (items > 0 && items < want) ns = (want + items - 1) / items;
        const int64_t cap = pl.max_key_tiles / 8;
        if (ns > cap) ns = cap;
        if (ns > kMaxSplits) ns = kMaxSplits;
        if (ns < 1) ns = 1;
        pl.nsplit = (int32_t)ns;
    }
    return pl;
}


// Launches the merge of nsplit partial results for n_rh (row, head) pairs.
void launch_merge(const AttnParams &p, int nsplit, hipStream_t hs)
{
    const int64_t n_rh = (int64_t)p.T * p.Hq;
    if (nsplit <= kMergeFewSplits) {
        const dim3 grid((unsigned)((n_rh + 7) / 8));
        if (nsplit <= 4)
            hipLaunchKernelGGL(merge_few_splits_kernel<4>, grid, dim3(256), 0, hs, p.part_o, p.part_ml, p.out, n_rh, nsplit);
        else
            hipLaunchKernelGGL(merge_few_splits_kernel<kMergeFewSplits>, grid, dim3(256), 0, hs, p.part_o, p.part_ml,
                               p.out, n_rh, nsplit);
    } else {
        hipLaunchKernelGGL(merge_splits_kernel, dim3((unsigned)n_rh), dim3(32 * kMergeGroups), 0, hs, p.part_o,
                           p.part_ml, p.out, n_rh, nsplit);
    }
}

size_t workspace_for(const cp_shape *s, const Plan &pl)
{
    if (pl.nsplit <= 1) return 0;
    const size_t rows = (size_t)pl.nsplit * (size_t)s->total_extend * (size_t)s->num_q_heads;
    size_t o_bytes = rows * kD * sizeof(float);
    size_t ml_bytes = rows * 2 * sizeof(float);
    return ((o_bytes + 255) / 256) * 256 + ((ml_bytes + 255) / 256) * 256;
}


inline bool aligned_to(const void *p, uintptr_t a) { return reinterpret_cast<uintptr_t>(p) % a == 0; }

// Device address of a file-scope __device__ array on the current device, looked up once per
// device (every device holds its own copy at its own address).
constexpr int kMaxDevices = 64;
struct SymbolCache {
    std::mutex lock;
    void *addr[kMaxDevices] = {};
};
template <typename Lookup>
void *device_address(SymbolCache &cache, Lookup lookup)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> guard(cache.lock);
    if (!cache.addr[dev]) {
        void *ptr = nullptr;
        if (lookup(&ptr) != hipSuccess) return nullptr;
        cache.addr[dev] = ptr;
    }
    return cache.addr[dev];
}
void *check_report_address()
{
    static SymbolCache cache;
    return device_address(cache, [](void **ptr) { return hipGetSymbolAddress(ptr, HIP_SYMBOL(g_check_report)); });
}

std::atomic<int> g_debug_validate{
#ifdef CP_DEBUG_VALIDATE
    1
#else
    -1 // not decided yet: the environment variable CP_DEBUG_VALIDATE is read on first use
#endif
};
bool debug_validate_on()
{
    int v = g_debug_validate.load(std::memory_order_relaxed);
    if (v < 0) {
        const char *e = getenv("CP_DEBUG_VALIDATE");
        v = (e && e[0] && e[0] != '0') ? 1 : 0;
        g_debug_validate.store(v, std::memory_order_relaxed);
    }
    return v == 1;
}

// The check itself: lengths are compared on the host after one copy, table entries on the
// device.  Waits for `stream` (this is the one place where the library synchronises).
int check_tables(const int32_t *block_table, const int32_t *prefix_lens, const int32_t *extend_lens,
                 hipStream_t hs, const cp_shape *s, int32_t *info)
{
    if (info) info[0] = info[1] = info[2] = -1;
    const int B = s->batch;
    std::vector<int32_t> dev_p((size_t)B), dev_e((size_t)B);
    if (hipMemcpyAsync(dev_p.data(), prefix_lens, (size_t)B * 4, hipMemcpyDeviceToHost, hs) != hipSuccess ||
        hipMemcpyAsync(dev_e.data(), extend_lens, (size_t)B * 4, hipMemcpyDeviceToHost, hs) != hipSuccess ||
        hipStreamSynchronize(hs) != hipSuccess)
        return CP_ERR_LAUNCH;
    for (int r = 0; r < B; ++r)
        if (dev_p[r] != s->h_prefix_lens[r] || dev_e[r] != s->h_extend_lens[r]) {
            if (info) {
                info[0] = r;
                info[1] = dev_p[r];
                info[2] = dev_e[r];
            }
            return CP_ERR_LENGTHS;
        }
    auto *report = static_cast<unsigned long long *>(check_report_address());
    if (!report) return CP_ERR_LAUNCH;
    const unsigned long long clear = ~0ull;
    if (hipMemcpyAsync(report, &clear, sizeof(clear), hipMemcpyHostToDevice, hs) != hipSuccess) return CP_ERR_LAUNCH;
    const int blocks_x = std::max(1, std::min(64, (s->max_pages_per_req + kCheckThreads - 1) / kCheckThreads));
    for (int r0 = 0; r0 < B; r0 += 65535) { // grid.y limit
        const int nb = std::min(65535, B - r0);
        hipLaunchKernelGGL(check_tables_kernel, dim3((unsigned)blocks_x, (unsigned)nb), dim3(kCheckThreads), 0, hs,
                           block_table + (int64_t)r0 * s->max_pages_per_req, prefix_lens + r0, extend_lens + r0, nb,
                           s->max_pages_per_req, s->num_pages, report);
        if (hipGetLastError() != hipSuccess) return CP_ERR_LAUNCH;
        unsigned long long got = 0;
        if (hipMemcpyAsync(&got, report, sizeof(got), hipMemcpyDeviceToHost, hs) != hipSuccess ||
            hipStreamSynchronize(hs) != hipSuccess)
            return CP_ERR_LAUNCH;
        if (got != ~0ull) {
            const bool bad_page = (got >> 62) != 0;
            const int r = r0 + (int)((got >> 31) & 0x7fffffffu), slot = (int)(got & 0x7fffffffu);
            int32_t entry = -1;
            if (bad_page && (hipMemcpyAsync(&entry, block_table + (int64_t)r * s->max_pages_per_req + slot, 4,
                                            hipMemcpyDeviceToHost, hs) != hipSuccess ||
                             hipStreamSynchronize(hs) != hipSuccess))
                return CP_ERR_LAUNCH;
            if (info) {
                info[0] = r;
                info[1] = bad_page ? slot : dev_p[r];
                info[2] = bad_page ? entry : dev_e[r];
            }
            return bad_page ? CP_ERR_TABLE : CP_ERR_LENGTHS;
        }
    }
    return CP_OK;
}

} // namespace

// Split-K / decode partial results of cp_extend_attention_noalloc: one array per device, held
// until the process ends.  Nothing in it has to start at zero (every partial that the merge
// reads is written by the launch before it), so it is never cleared; calls that overlap on one
// device share it and race.
#define CP_NOALLOC_SCRATCH_BYTES (64u << 20)
static __device__ __align__(256) unsigned char scratch[CP_NOALLOC_SCRATCH_BYTES];

namespace {
void *scratch_address()
{
    static SymbolCache cache;
    return device_address(cache, [](void **ptr) { return hipGetSymbolAddress(ptr, HIP_SYMBOL(scratch)); });
}
} // namespace

extern "C" {

const char *cp_status_string(int status)
{
    switch (status) {
    case CP_OK: return "ok";
    case CP_ERR_NULL: return "a required pointer is NULL";
    case CP_ERR_SHAPE: return "unsupported or inconsistent shape";
    case CP_ERR_WORKSPACE:
        return "workspace missing, too small or misaligned (cp_extend_attention_noalloc: the shape needs more "
               "than the library's own scratch)";
    case CP_ERR_LAUNCH: return "HIP launch error";
    case CP_ERR_ALIGN: return "a device pointer is not aligned as required";
    case CP_ERR_TABLE: return "block_table holds a page id outside [0, num_pages)";
    case CP_ERR_LENGTHS: return "device prefix_lens / extend_lens differ from the host copies";
    default: return "unknown status";
    }
}

int32_t cp_num_splits(const cp_shape *shape)
{
    if (validate(shape) != CP_OK) return 0;
    return make_plan(shape).nsplit;
}

int32_t cp_plan_kind(const cp_shape *shape)
{
    if (validate(shape) != CP_OK) return CP_PLAN_INVALID;
    const Plan pl = make_plan(shape);
    if (pl.decode) return CP_PLAN_DECODE;
    return pl.nsplit > 1 ? CP_PLAN_ROW_TILED_SPLIT : CP_PLAN_ROW_TILED;
}

size_t cp_workspace_bytes(const cp_shape *shape)
{
    if (validate(shape) != CP_OK) return 0;
    return workspace_for(shape, make_plan(shape));
}

} // extern "C"

namespace {
// Everything behind cp_extend_attention: argument checks, plan, launches.  `workspace` is
// whatever scratch the entry point brings: the caller's buffer or the library's own array.
int run_attention(const void *q, const void *k_new, const void *v_new, const void *kv_pages,
                  const int32_t *block_table, const int32_t *prefix_lens, const int32_t *extend_lens, void *out,
                  void *stream, const cp_shape *shape, void *workspace, size_t workspace_bytes)
{
    const int st = validate(shape);
    if (st != CP_OK) return st;
    if (!block_table || !prefix_lens || !extend_lens) return CP_ERR_NULL;
    if (shape->total_extend == 0) return CP_OK;
    if (!q || !k_new || !v_new || !kv_pages || !out) return CP_ERR_NULL;
    if (!aligned_to(q, 16) || !aligned_to(k_new, 16) || !aligned_to(v_new, 16) || !aligned_to(kv_pages, 16) ||
        !aligned_to(out, 16) || !aligned_to(block_table, 4) || !aligned_to(prefix_lens, 4) ||
        !aligned_to(extend_lens, 4))
        return CP_ERR_ALIGN;
    if (debug_validate_on()) {
        const int chk = check_tables(block_table, prefix_lens, extend_lens, static_cast<hipStream_t>(stream), shape,
                                     nullptr);
        if (chk != CP_OK) return chk;
    }
    const Plan pl = make_plan(shape);
    const size_t need = workspace_for(shape, pl);
    if (need > 0) {
        if (!workspace || workspace_bytes < need) return CP_ERR_WORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return CP_ERR_WORKSPACE;
    }
    const int64_t per_head = pl.q_tiles * pl.nsplit;
    const int64_t total = per_head * shape->num_kv_heads;
    if (total > INT32_MAX / 2) return CP_ERR_SHAPE;
    const int64_t dec_units = (int64_t)shape->batch * shape->num_kv_heads * pl.nsplit * pl.row_blocks;
    if (pl.decode && dec_units > INT32_MAX / 2) return CP_ERR_SHAPE;

    AttnParams p;
    p.q = static_cast<const uint16_t *>(q);
    p.k_new = static_cast<const uint16_t *>(k_new);
    p.v_new = static_cast<const uint16_t *>(v_new);
    p.kv_pages = static_cast<const uint16_t *>(kv_pages);
    p.block_table = block_table;
    p.prefix_lens = prefix_lens;
    p.extend_lens = extend_lens;
    p.out = static_cast<uint16_t *>(out);
    p.part_o = nullptr;
    p.part_ml = nullptr;
    p.batch = shape->batch;
    p.Hq = shape->num_q_heads;
    p.Hkv = shape->num_kv_heads;
    p.G = shape->num_q_heads / shape->num_kv_heads;
    p.max_pages = shape->max_pages_per_req;
    p.T = shape->total_extend;
    p.nsplit = pl.nsplit;
    p.dec_row_blocks = pl.row_blocks;
    p.items_per_head = (int32_t)per_head;
    p.total_items = (int32_t)total;
    p.items_per_xcd = (int32_t)((total + kXcds - 1) / kXcds);
    p.scale_log2 = shape->softmax_scale * 1.4426950408889634f;

    hipStream_t hs = static_cast<hipStream_t>(stream);
    if (pl.decode) {
        const size_t rows = (size_t)pl.nsplit * (size_t)p.T * (size_t)p.Hq;
        const size_t o_bytes = ((rows * kD * sizeof(float) + 255) / 256) * 256;
        p.part_o = static_cast<float *>(workspace);
        p.part_ml = reinterpret_cast<float *>(static_cast<char *>(workspace) + o_bytes);
        hipLaunchKernelGGL(decode_attn_kernel, dim3((unsigned)(dec_units / kDecWaves)), dim3(kDecWaves * 64), 0, hs, p);
        if (hipGetLastError() != hipSuccess) return CP_ERR_LAUNCH;
        launch_merge(p, pl.nsplit, hs);
        return hipGetLastError() == hipSuccess ? CP_OK : CP_ERR_LAUNCH;
    }
    if (!allow_large_lds()) return CP_ERR_LAUNCH;
    const dim3 grid((unsigned)(p.items_per_xcd * kXcds)), block(kThreads);
    if (pl.nsplit > 1) {
        const size_t rows = (size_t)pl.nsplit * (size_t)p.T * (size_t)p.Hq;
        const size_t o_bytes = ((rows * kD * sizeof(float) + 255) / 256) * 256;
        p.part_o = static_cast<float *>(workspace);
        p.part_ml = reinterpret_cast<float *>(static_cast<char *>(workspace) + o_bytes);
        hipLaunchKernelGGL(extend_attn_kernel<true>, grid, block, kLdsBytes, hs, p);
        if (hipGetLastError() != hipSuccess) return CP_ERR_LAUNCH;
        launch_merge(p, pl.nsplit, hs);
    } else {
        hipLaunchKernelGGL(extend_attn_kernel<false>, grid, block, kLdsBytes, hs, p);
    }
    if (hipGetLastError() != hipSuccess) return CP_ERR_LAUNCH;
    return CP_OK;
}
} // namespace

extern "C" {

int cp_extend_attention(const void *q, const void *k_new, const void *v_new, const void *kv_pages,
                        const int32_t *block_table, const int32_t *prefix_lens,
                        const int32_t *extend_lens, void *out, void *stream, const cp_shape *shape,
                        void *workspace, size_t workspace_bytes)
{
    return run_attention(q, k_new, v_new, kv_pages, block_table, prefix_lens, extend_lens, out, stream, shape,
                         workspace, workspace_bytes);
}

size_t cp_noalloc_scratch_bytes(void) { return CP_NOALLOC_SCRATCH_BYTES; }

int cp_extend_attention_noalloc(const void *q, const void *k_new, const void *v_new, const void *kv_pages,
                                const int32_t *block_table, const int32_t *prefix_lens,
                                const int32_t *extend_lens, void *out, void *stream, const cp_shape *shape)
{
    const int st = validate(shape);
    if (st != CP_OK) return st;
    // sizes beyond the library's own array are refused here, before anything is looked up or launched
    if (workspace_for(shape, make_plan(shape)) > CP_NOALLOC_SCRATCH_BYTES) return CP_ERR_WORKSPACE;
    void *ptr = scratch_address(); // the array's address on the current device, never the array's name
    if (!ptr) return CP_ERR_LAUNCH;
    return run_attention(q, k_new, v_new, kv_pages, block_table, prefix_lens, extend_lens, out, stream, shape, ptr,
                         CP_NOALLOC_SCRATCH_BYTES);
}

int cp_write_kv(const void *k_new, const void *v_new, void *kv_pages, const int32_t *block_table,
                const int32_t *prefix_lens, const int32_t *extend_lens, void *stream,
                const cp_shape *shape)
{
    const int st = validate(shape);
    if (st != CP_OK) return st;
    if (!block_table || !prefix_lens || !extend_lens) return CP_ERR_NULL;
    if (shape->total_extend == 0) return CP_OK;
    if (!k_new || !v_new || !kv_pages) return CP_ERR_NULL;
    if (!aligned_to(k_new, 16) || !aligned_to(v_new, 16) || !aligned_to(kv_pages, 16) ||
        !aligned_to(block_table, 4) || !aligned_to(prefix_lens, 4) || !aligned_to(extend_lens, 4))
        return CP_ERR_ALIGN;
    if (debug_validate_on()) {
        const int chk = check_tables(block_table, prefix_lens, extend_lens, static_cast<hipStream_t>(stream), shape,
                                     nullptr);
        if (chk != CP_OK) return chk;
    }
    const int T = shape->total_extend;
    const dim3 grid((unsigned)((T + kWriteRows - 1) / kWriteRows)), block(256);
    hipLaunchKernelGGL(write_kv_kernel, grid, block, 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint16_t *>(k_new), static_cast<const uint16_t *>(v_new),
                       static_cast<uint16_t *>(kv_pages), block_table, prefix_lens, extend_lens,
                       shape->batch, shape->num_kv_heads, shape->max_pages_per_req, T);
    if (hipGetLastError() != hipSuccess) return CP_ERR_LAUNCH;
    return CP_OK;
}

int cp_check_tables(const int32_t *block_table, const int32_t *prefix_lens, const int32_t *extend_lens,
                    void *stream, const cp_shape *shape, int32_t *info)
{
    const int st = validate(shape);
    if (st != CP_OK) return st;
    if (!block_table || !prefix_lens || !extend_lens) return CP_ERR_NULL;
    if (!aligned_to(block_table, 4) || !aligned_to(prefix_lens, 4) || !aligned_to(extend_lens, 4)) return CP_ERR_ALIGN;
    return check_tables(block_table, prefix_lens, extend_lens, static_cast<hipStream_t>(stream), shape, info);
}

void cp_set_debug_validate(int on) { g_debug_validate.store(on ? 1 : 0, std::memory_order_relaxed); }

} // extern "C"
