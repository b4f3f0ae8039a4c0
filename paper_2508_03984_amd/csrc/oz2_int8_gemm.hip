// Batched INT8 GEMM with exact (wrapping) INT32 accumulation on the gfx950 matrix cores:
// Algorithm 1 line 6, C'_s = A'_s B'_s for all moduli s in one launch.
//
// Operands are the padded residue slices in the K-blocked layout the residue kernel
// writes: A [batch][Kp/64][Mp][64] and B [batch][Kp/64][Np][64] (B transposed), i.e. 64
// consecutive k of one row are contiguous and consecutive rows of one 64-wide K block
// follow each other.  A (rows x 64) tile of either operand is then one contiguous run of
// memory, fetched as whole 128-byte lines, both tiles are staged through LDS the same way
// and every MFMA operand is a 16-byte K-run read with one ds_read_b128.
//
// Tiling: workgroup = WM x WN wavefronts, block tile (32 TM WM) x (32 TN WN) x 64, each
// wavefront owns (32 TM) x (32 TN) = TM x TN v_mfma_i32_32x32x32_i8 accumulators.  The
// large configuration is 2 x 4 wavefronts of 128 x 64 (a 256 x 256 block, 128 accumulator
// registers per lane, two wavefronts per SIMD).
//
// Data movement: global_load_lds_dwordx4 copies HBM/L2 straight into a ring of STAGES LDS
// stages, STAGES-1 tiles ahead of the math, so no VGPRs or ds_write instructions are spent
// on staging.  A wavefront's 64 lanes fill 64 consecutive 16-byte LDS chunks per
// instruction; the XOR swizzle that keeps the fragment reads free of bank conflicts is
// applied on the global side (which 16 bytes of a row a lane fetches).  MFMA operands are
// double-buffered in registers and fetched one 32-deep K step ahead, across stage
// boundaries, so LDS latency is covered by 16 MFMAs.
//
// Synchronisation per K tile: one s_waitcnt vmcnt(n) that leaves the youngest tiles in
// flight, then one s_barrier.  The compiler does not track LDS writes made by
// global_load_lds, so these two are what orders them against the ds_reads.
#include <algorithm>
#include <type_traits>

#include "oz2_kernels.hpp"

namespace oz2 {
namespace {

constexpr int64_t kMaxExactK = (int64_t)1 << 17;   // Section 4.3: no INT32 overflow up to here
#ifndef OZ2_PERSISTENT_MAX_K
#define OZ2_PERSISTENT_MAX_K 4096
#endif
constexpr int64_t kPersistentMaxK = OZ2_PERSISTENT_MAX_K;   // contractions up to here run as a persistent grid

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef const __attribute__((address_space(1))) void *global_ptr_t;

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and
// 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima).
constexpr int vmcnt_imm(int n) { return (n & 0xf) | ((n >> 4) << 14) | (0x7 << 4) | (0xf << 8); }

// LDS on this chip is 64 banks x 4 B: a 256-byte line is 16 slots of 16 B, and a
// ds_read_b128 is served 16 lanes per clock.  A tile row is CPR slots, so rows r and
// r + 16/CPR start in the same slot; XOR-ing the chunk index with (row / (16/CPR)) spreads
// the 32 rows that a fragment read touches over all 16 slots in every group of lanes the
// hardware serves together (measured: 230 B/clk/CU against 125 with a 128-byte-line swizzle).
template <int CPR>
__device__ inline int swizzle_mask(int row) {
    return (row / (16 / CPR)) & (CPR - 1);
}

struct TileMap {
    int tiles_m, tiles_n;      // tiles per slice
    int swizzled;              // 1: tiles_m and tiles_n are multiples of 16
};

// Workgroup id -> (slice, tile row, tile column).  Workgroups are handed to the 8 XCDs
// round-robin by id, and 256 run at a time (one per CU).  In the swizzled map the 256
// co-resident workgroups cover one 16 x 16-tile region of one slice, and the 32 that share
// an XCD (and its L2) cover an 8 x 4 sub-block of it, so an A tile row is fetched into that
// L2 once for 4 workgroups and a B tile row once for 8.
__device__ inline void map_tile(const TileMap &tm, int id, int &s, int &tr, int &tc) {
    if (tm.swizzled) {
        const int xcd = id & 7, local = id >> 3;
        const int pos = local & 31, region = local >> 5;
        const int regions_n = tm.tiles_n / 16, regions = (tm.tiles_m / 16) * regions_n;
        s = region / regions;
        const int r = region % regions;
        tr = (r / regions_n) * 16 + (xcd >> 2) * 8 + (pos >> 2);
        tc = (r % regions_n) * 16 + (xcd & 3) * 4 + (pos & 3);
    } else {
        const int per = tm.tiles_m * tm.tiles_n;
        s = id / per;
        tr = (id % per) / tm.tiles_n;
        tc = id % tm.tiles_n;
    }
}

// What the store phase writes (Algorithm 1 lines 6-7):
//   kOutI32      C'_s as int32 (diagnostics: the raw products)
//   kOutI32Fold  int32: mod(old, p_s) + mod(C'_s, p_s)   (a further K range of a k > 2^17 product)
//   kOutU8       U_s = mod(C'_s, p_s) as uint8 -- the form the accumulation kernel wants
//   kOutU8Fold   uint8: (old + mod(C'_s, p_s)) mod p_s
//   kOutMax      nothing of the product itself: only its row and column maxima, folded into
//                two int arrays with atomic maxima (accurate mode of Section 4.2, where the
//                product Cbar = Abar * Bbar of the 7-bit matrices is needed for nothing else).
//                The kernel arguments then mean: C = the row maxima of the panel's rows,
//                C + c_plane (in ints) = the column maxima of its columns, c_ld = the number of
//                valid rows of the panel in its low and of valid columns in its high 32 bits.
//                (k_int8_gemm only.)
enum { kOutI32 = 0, kOutI32Fold = 1, kOutU8 = 2, kOutU8Fold = 3, kOutMax = 4 };

// (a + b) mod p on each of the four bytes of a and b, all of them below p <= 256: the even and
// the odd bytes as two pairs of 16-bit sums (at most 510), each reduced by one packed unsigned
// minimum (s - p wraps to a large number when s < p).
typedef unsigned short us2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t add_mod_bytes(uint32_t a, uint32_t b, int p) {
    const us2 pp = {(unsigned short)p, (unsigned short)p};
    auto reduce = [&](uint32_t x) {
        const us2 v = __builtin_bit_cast(us2, x);
        return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(v, (us2)(v - pp)));
    };
    const uint32_t even = reduce((a & 0x00ff00ffu) + (b & 0x00ff00ffu));
    const uint32_t odd = reduce(((a >> 8) & 0x00ff00ffu) + ((b >> 8) & 0x00ff00ffu));
    return even | (odd << 8);
}

struct GemmMods {                       // moduli of the slices and their mulhi multipliers
    int32_t p[kMaxModuli];
    int32_t pinv_prime[kMaxModuli];
};

// The LDS of a workgroup: STAGES stages of (A rows | B rows) x 64 bytes.  Declared here, not
// passed around, so that every access is an offset from a base the compiler knows.
extern __shared__ v4i lds[];                              // [STAGES][ROWS][CPR]

// Everything one workgroup does for one output tile, shared by the two kernels below: where its
// lanes fetch from, the K loop, and the store phase.  A tile is identified by the global address
// its loads start at (tile_source) and by (slice, first row, first column) for the store.
template <int WM, int WN, int TM, int TN, int BK, int STAGES>
struct GemmCore {
    static constexpr int THREADS = 64 * WM * WN;              // WM x WN wavefronts
    static constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    static constexpr int CPR = BK / 16;                       // 16-byte chunks per tile row
    static constexpr int ROWS = BM + BN;                      // A rows then B rows in one LDS stage
    static constexpr int CHUNKS = ROWS * CPR;
    static constexpr int LPT = CHUNKS / THREADS;              // LDS-direct loads per lane and tile
    static constexpr int KK = BK / 32;                        // MFMA K steps per tile
    static constexpr int STAGE_BYTES = CHUNKS * 16;
    static constexpr int ROWS_PER_LOAD = 64 / CPR;            // rows one wavefront-wide load covers
    static constexpr int SRC_STEP = ROWS_PER_LOAD * BK;
    static_assert(CHUNKS % THREADS == 0 && (BM * CPR) % (64 * LPT) == 0,
                  "each wavefront must load from one operand only");
    static_assert(BK == kBlockK, "the K tile is the K block of the operand layout");
    static_assert(CPR == 4, "the load-side swizzle below assumes one mask per lane");
    static_assert(STAGES >= 3 && (STAGES - 3) * LPT < 64, "vmcnt is a 6-bit counter");
    static_assert(KK >= 2, "operand double-buffering assumes an even number of K steps");

    int wm, wn, lrow, lhalf;
    // Load i of this wavefront fills LDS chunks [64 q, 64 q + 64) of a stage, q = wave*LPT + i,
    // i.e. rows q*ROWS_PER_LOAD ...; lane -> (row, physical chunk) -> logical chunk to fetch.
    // In the blocked layout those 64 chunks are 1 KiB of contiguous memory, so the LPT loads of a
    // wavefront and tile differ by i KiB in the global AND in the LDS address: one address and
    // one LDS base (M0) per tile, the rest is the instruction's immediate offset, which the
    // hardware applies to both.
    static_assert(ROWS_PER_LOAD * BK == 1024 && (LPT - 1) * 1024 < 4096, "immediate offset of the loads");
    int row0, ch;
    bool from_a;                                              // uniform over the wavefront
    int64_t tile_step;                                        // next K block of the same rows
    int my_dst;                                               // uniform: byte offset within a stage
    // Fragment addressing: lane l reads row (l % 32) of a 32-row fragment, 16-byte chunk
    // 2*kk + l/32 of the K tile.  The swizzle mask depends on l % 32 only.
    int a_addr[KK], b_addr[KK];                               // byte offsets within a stage, per K step

    __device__ __forceinline__ GemmCore(int64_t Mp, int64_t Np) {
        const int tid = threadIdx.x, lane = tid & 63;
        // the wavefront index as a scalar: everything derived from it stays in scalar registers
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        wm = wave / WN; wn = wave % WN;
        const int row0u = wave * LPT * ROWS_PER_LOAD;
        row0 = row0u + lane / CPR;
        ch = (lane % CPR) ^ swizzle_mask<CPR>(row0);
        from_a = row0u < BM;
        tile_step = (from_a ? Mp : Np) * BK;
        my_dst = wave * LPT * 1024;
        lrow = lane & 31; lhalf = lane >> 5;
        const int mask = swizzle_mask<CPR>(lrow);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const int c = (kk * 2 + lhalf) ^ mask;
            a_addr[kk] = ((wm * 32 * TM + lrow) * CPR + c) * 16;
            b_addr[kk] = ((BM + wn * 32 * TN + lrow) * CPR + c) * 16;
        }
    }

    // Where this lane's loads of tile (s, tr, tc) start.  KB = K blocks per slice; the launch
    // contracts over blocks [kb0, kb0 + KT).
    __device__ __forceinline__ const int8_t *tile_source(const int8_t *A, const int8_t *B, int s, int tr, int tc,
                                                         int64_t Mp, int64_t Np, int64_t KB, int kb0) const {
        const int8_t *Ab = A + (((int64_t)s * KB + kb0) * Mp + (int64_t)tr * BM) * BK;
        const int8_t *Bb = B + (((int64_t)s * KB + kb0) * Np + (int64_t)tc * BN) * BK;
        return (from_a ? Ab + (int64_t)row0 * BK : Bb + (int64_t)(row0 - BM) * BK) + ch * 16;
    }

    // Loads [I0, I1) of the K tile whose loads start at src_t, into the stage at byte offset
    // stage_off (uniform).
    template <int I0, int I1>
    __device__ __forceinline__ void issue_loads(const int8_t *src_t, int stage_off) const {
        if constexpr (I0 < I1) {
            __builtin_amdgcn_global_load_lds((global_ptr_t)src_t,
                                             (lds_ptr_t)(reinterpret_cast<char *>(lds) + stage_off + my_dst), 16,
                                             I0 * 1024, 0);
            issue_loads<I0 + 1, I1>(src_t, stage_off);
        }
    }

    // The first STAGES - 1 K tiles of a tile.  KT >= 2: every K range is a multiple of 128.
    __device__ __forceinline__ void issue_head(const int8_t *src_tile, int KT) const {
#pragma unroll
        for (int t = 0; t < STAGES - 1; ++t)
            if (t < KT) issue_loads<0, LPT>(src_tile + (int64_t)t * tile_step, t * STAGE_BYTES);
    }

    // The K loop over a tile whose head has been requested: acc += A tile * B tile^T.
    // It is written so that the instruction stream between the MFMAs stays as short as it can be:
    // the loop is split into iterations that prefetch (all but the last STAGES - 1) and ones that
    // do not, so there is no branch per load; the LDS stage offsets are carried along, not
    // recomputed (measured against the same pipeline with a branch and a readfirstlane per load:
    // 3.5 % faster at 16 x 4096 x 4096 x 16384).
    __device__ __forceinline__ void contract(const int8_t *src_tile, int KT, v16i (&acc)[TM][TN]) const {
        v4i fa[2][TM], fb[2][TN];
        const char *const lds_bytes = reinterpret_cast<const char *>(lds);
        auto load_frags = [&](int buf, int stage_off, int kk) {
            const char *st = lds_bytes + stage_off;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[buf][i] = *reinterpret_cast<const v4i *>(st + a_addr[kk] + i * 32 * CPR * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[buf][j] = *reinterpret_cast<const v4i *>(st + b_addr[kk] + j * 32 * CPR * 16);
        };

        // K tiles 0 and 1 must have landed before the first fragment reads.  (In the persistent
        // kernel the stores of this workgroup's previous tile are outstanding as well; they were
        // issued after these loads, and loads complete in order, so "at most the youngest K tile
        // outstanding" still implies that K tiles 0 and 1 are complete.)
        if (KT >= STAGES - 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm((STAGES - 3) * LPT));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        __builtin_amdgcn_s_barrier();
        load_frags(0, 0, 0);

        // One K tile: it is read from the stage at cur_off, the K tile STAGES - 1 ahead is
        // requested into the stage read during the previous iteration.  Its LPT loads go out in
        // two halves, each behind the second MFMA row of a K step.
        int cur_off = 0;
        const int8_t *src_ld = src_tile + (int64_t)(STAGES - 1) * tile_step;
        auto iteration = [&](auto issued_c, bool last) {
            constexpr bool issued = decltype(issued_c)::value;
            const int nxt_off = cur_off + STAGE_BYTES == STAGES * STAGE_BYTES ? 0 : cur_off + STAGE_BYTES;
            const int ld_off = cur_off == 0 ? (STAGES - 1) * STAGE_BYTES : cur_off - STAGE_BYTES;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const int cur = kk & 1, nxt = cur ^ 1;
                // The first MFMA row runs before the next operands are requested: its operands
                // were requested a whole K step ago, so waiting for them (the LDS counter is
                // waited down to zero at that point) does not wait for the new requests.
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[0][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[cur][j], fa[cur][0], acc[0][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (kk + 1 < KK) load_frags(nxt, cur_off, kk + 1);
                else if (!last) load_frags(nxt, nxt_off, 0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 1; i < TM; ++i) {
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    if (issued && i == 1) {
                        if (kk == 0) issue_loads<0, LPT / 2>(src_ld, ld_off);
                        if (kk == KK - 1) issue_loads<LPT / 2, LPT>(src_ld, ld_off);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // Tile kt + 2 must be complete (and visible to every wavefront) before iteration
            // kt + 1 prefetches fragments from it; the barrier also frees the stage just read.
            if (issued) __builtin_amdgcn_s_waitcnt(vmcnt_imm((STAGES - 3) * LPT));
            else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            __builtin_amdgcn_s_barrier();
            cur_off = nxt_off;
            src_ld += tile_step;
        };
        int kt = 0;
        for (; kt + STAGES - 1 < KT; ++kt) iteration(std::true_type{}, false);
        for (; kt < KT; ++kt) iteration(std::false_type{}, kt + 1 == KT);
    }

    // Row and column maxima of the tile (kOutMax).  Entries are sums of products of non-negative
    // 7-bit numbers (k <= 2^17: below 2^29), the maxima start at 0 and zero entries (all the
    // padding) are skipped, so integer atomic maxima give the exact result whatever the order.  A
    // lane holds, per 32 x 32 block, 16 columns of one row: the row maximum is completed by the
    // lane 32 further on, a column maximum by the 32 lanes of the same half-wavefront.
    __device__ __forceinline__ void store_maxima(const v16i (&acc)[TM][TN], int *rmax, int *cmax, int64_t bm,
                                                 int64_t bn, int valid_rows, int valid_cols) const {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            int v = 0;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) v = acc[i][j][r] > v ? acc[i][j][r] : v;
            const int o = __shfl_xor(v, 32, 64);
            v = o > v ? o : v;
            const int row = (int)bm + wm * 32 * TM + i * 32 + lrow;
            if (lhalf == 0 && v > 0 && row < valid_rows) atomicMax(&rmax[row], v);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int v = 0;
#pragma unroll
                for (int i = 0; i < TM; ++i) v = acc[i][j][r] > v ? acc[i][j][r] : v;
#pragma unroll
                for (int off = 1; off < 32; off <<= 1) {
                    const int o = __shfl_xor(v, off, 64);
                    v = o > v ? o : v;
                }
                const int col = (int)bn + wn * 32 * TN + j * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                if (lrow == 0 && v > 0 && col < valid_cols) atomicMax(&cmax[col], v);
            }
    }

    // The store phase (Algorithm 1 lines 6-7 in the forms listed at kOut...).  The B fragment is
    // the MFMA's first operand, so the 32x32 accumulator is the transposed block: lane l holds
    // row (l % 32) of the C block and, in registers 4g .. 4g+3, the four consecutive columns
    // 8g + 4*(l / 32) + {0,1,2,3}.  The reduction is the mulhi form of Section 4.3 (an FP64
    // floor/fma version measured 1.1 ms slower per launch at 16 x 16384^3).
    template <int OUT>
    __device__ __forceinline__ void store(const v16i (&acc)[TM][TN], void *C, int s, int64_t bm, int64_t bn,
                                          int64_t c_ld, int64_t c_plane, const GemmMods &mods) const {
        const int p = mods.p[s], pv = mods.pinv_prime[s];
        const int64_t c_off = (int64_t)s * c_plane + bm * c_ld + bn;   // C: [slice][row][column]
        if (OUT == kOutU8 || OUT == kOutU8Fold) {
            // Four residues per register quad pack into one dword; the two half-wavefronts hold
            // alternating dwords of a row (columns 8g + 4*(l/32) ...), so they swap two dwords
            // each (lanes 0-31 end up with columns 0-15 of the block row, lanes 32-63 with 16-31)
            // and every lane stores 16 contiguous bytes: a lane pair completes a 32-byte
            // sector of the row, and the L2 does not have to fetch lines to merge 4-byte stores.
            // (Staging the whole uint8 tile through LDS to store 64-byte row segments was measured
            // 3.5 ms slower per launch at 16 x 16384^3.)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    uint32_t d[4];
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        d[g] = 0;
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            d[g] |= (uint32_t)mod_small(acc[i][j][4 * g + c], p, pv) << (8 * c);
                    }
                    // v_permlane32_swap(a, b): the upper half of a and the lower half of b change
                    // places, so lanes 0-31 get (d0 | d0 of lane + 32) and lanes 32-63 (d2 of lane
                    // - 32 | d2) in (a, b): the row's dwords in column order, no selects needed.
                    const auto s0 = __builtin_amdgcn_permlane32_swap(d[0], d[2], false, false);
                    const auto s1 = __builtin_amdgcn_permlane32_swap(d[1], d[3], false, false);
                    v4i q = v4i{(int)s0[0], (int)s0[1], (int)s1[0], (int)s1[1]};
                    const int row = wm * 32 * TM + i * 32 + lrow;
                    const int col = wn * 32 * TN + j * 32 + 16 * lhalf;
                    v4i *dst = reinterpret_cast<v4i *>(static_cast<uint8_t *>(C) + c_off + (int64_t)row * c_ld + col);
                    if (OUT == kOutU8Fold) {               // a further K range: (old + new) mod p_s, byte by byte
                        const v4i old = *dst;
#pragma unroll
                        for (int w = 0; w < 4; ++w) q[w] = (int)add_mod_bytes((uint32_t)q[w], (uint32_t)old[w], p);
                    }
                    *dst = q;
                }
            return;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int row = wm * 32 * TM + i * 32 + lrow;
                    const int col = wn * 32 * TN + j * 32 + 8 * g + 4 * lhalf;
                    const int64_t at = c_off + (int64_t)row * c_ld + col;
                    int v[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) v[c] = acc[i][j][4 * g + c];
                    v4i *dst = reinterpret_cast<v4i *>(static_cast<int32_t *>(C) + at);
                    if (OUT == kOutI32Fold) {
                        const v4i old = *dst;
#pragma unroll
                        for (int c = 0; c < 4; ++c) v[c] = mod_small(old[c], p, pv) + mod_small(v[c], p, pv);
                    }
                    *dst = v4i{v[0], v[1], v[2], v[3]};
                }
    }

    static __device__ __forceinline__ void clear(v16i (&acc)[TM][TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    }
};

// One workgroup per output tile.  For kOutMax the arguments mean: C = the row maxima of the
// panel's rows, C + c_plane (in ints) = the column maxima of its columns, c_ld = the number of
// valid rows of the panel in its low and of valid columns in its high 32 bits.
template <int WM, int WN, int TM, int TN, int BK, int STAGES, int OUT>
__global__ __launch_bounds__(64 * WM * WN) void k_int8_gemm(const int8_t *__restrict__ A,
                                                   const int8_t *__restrict__ B,
                                                   void *__restrict__ C, int64_t Mp,
                                                   int64_t Np, int64_t KB, int kb0, int KT,
                                                   int64_t c_ld, int64_t c_plane,
                                                   TileMap tmap, GemmMods mods) {
    typedef GemmCore<WM, WN, TM, TN, BK, STAGES> Core;
    const Core core(Mp, Np);
    int s, tile_r, tile_c;
    map_tile(tmap, (int)blockIdx.x, s, tile_r, tile_c);
    const int8_t *src = core.tile_source(A, B, s, tile_r, tile_c, Mp, Np, KB, kb0);
    core.issue_head(src, KT);
    v16i acc[TM][TN];
    Core::clear(acc);
    core.contract(src, KT, acc);
    const int64_t bm = (int64_t)tile_r * Core::BM, bn = (int64_t)tile_c * Core::BN;
    if (OUT == kOutMax) {
        int *rmax = static_cast<int *>(C);
        core.store_maxima(acc, rmax, rmax + c_plane, bm, bn, (int)(c_ld & 0xffffffff), (int)(c_ld >> 32));
    } else {
        core.template store<OUT>(acc, C, s, bm, bn, c_ld, c_plane, mods);
    }
}

// The same as a persistent grid, for short contractions: as many workgroups as compute units,
// each walking over the tiles id = blockIdx.x, blockIdx.x + gridDim.x, ...  The head of the next
// tile (its first STAGES - 1 K tiles) is requested before the results of the last one are
// reduced and stored, and no workgroup is dispatched per tile.  With a short k a tile is a few
// microseconds of matrix-core work, so that the dispatch between tiles and the wait for the
// first operands weigh as much as the contraction (16384 x 16384 x 512, N = 15: 3.84 -> 3.09 ms;
// 2048^3, N = 14: 2.5 % faster).  For long contractions the two forms take the same time (the
// store phase, which nothing overlaps in either form, is what a tile costs beyond its K loop),
// so the plain one-workgroup-per-tile kernel is kept there.
template <int WM, int WN, int TM, int TN, int BK, int STAGES, int OUT>
__global__ __launch_bounds__(64 * WM * WN) void k_int8_gemm_persistent(const int8_t *__restrict__ A,
                                                   const int8_t *__restrict__ B,
                                                   void *__restrict__ C, int64_t Mp,
                                                   int64_t Np, int64_t KB, int kb0, int KT,
                                                   int64_t c_ld, int64_t c_plane,
                                                   TileMap tmap, int total_tiles, GemmMods mods) {
    typedef GemmCore<WM, WN, TM, TN, BK, STAGES> Core;
    static_assert(OUT != kOutMax, "the maxima form runs one workgroup per tile");
    const Core core(Mp, Np);
    int tile = (int)blockIdx.x;
    int s, tile_r, tile_c;
    map_tile(tmap, tile, s, tile_r, tile_c);
    const int8_t *src = core.tile_source(A, B, s, tile_r, tile_c, Mp, Np, KB, kb0);
    core.issue_head(src, KT);
    for (;;) {
        v16i acc[TM][TN];
        Core::clear(acc);
        core.contract(src, KT, acc);
        // Every wavefront has passed the last barrier, so nothing reads the LDS stages any more:
        // the head of this workgroup's next tile is requested now and travels while the results
        // of this one are reduced and stored.
        const int next = tile + (int)gridDim.x;
        int s_next = 0, tile_r_next = 0, tile_c_next = 0;
        const int8_t *src_next = nullptr;
        if (next < total_tiles) {
            map_tile(tmap, next, s_next, tile_r_next, tile_c_next);
            src_next = core.tile_source(A, B, s_next, tile_r_next, tile_c_next, Mp, Np, KB, kb0);
            core.issue_head(src_next, KT);
        }
        core.template store<OUT>(acc, C, s, (int64_t)tile_r * Core::BM, (int64_t)tile_c * Core::BN, c_ld, c_plane,
                                 mods);
        if (next >= total_tiles) break;                    // uniform over the workgroup
        tile = next; s = s_next; tile_r = tile_r_next; tile_c = tile_c_next; src = src_next;
    }
}

// Compute units of the current device (cached per device id).
int compute_units() {
    static thread_local int cached_dev = -1, cached = 0;     // contexts may launch from several threads
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (dev != cached_dev) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
        cached = n; cached_dev = dev;
    }
    return cached;
}

template <int WM, int WN, int TM, int TN, int BK, int STAGES, int OUT>
hipError_t launch_persistent(const int8_t *A, const int8_t *B, void *C, int batch, int64_t Mp, int64_t Np,
                             int64_t Kp, int64_t k_begin, int64_t k_len, const GemmPanel &pn,
                             const GemmMods &mods, hipStream_t stream) {
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    constexpr size_t lds_bytes = (size_t)STAGES * (BM + BN) * BK;
    static_assert(lds_bytes > 80 * 1024, "one workgroup per compute unit is assumed");
    static thread_local int attr_device = -1;                // the attribute is per device (set again per thread: harmless)
    int dev = -1;
    if (hipError_t e = hipGetDevice(&dev)) return e;
    if (attr_device != dev) {
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void *>(&k_int8_gemm_persistent<WM, WN, TM, TN, BK, STAGES, OUT>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_device = dev;
    }
    TileMap tm;
    tm.tiles_m = (int)(pn.rows / BM);
    tm.tiles_n = (int)(pn.cols / BN);
    tm.swizzled = (tm.tiles_m % 16 == 0 && tm.tiles_n % 16 == 0) ? 1 : 0;
    const int64_t total = (int64_t)tm.tiles_m * tm.tiles_n * batch;
    if (total > 0x7fff0000) return hipErrorInvalidValue;      // tile ids (plus one grid stride) fit an int
    // The grid is a multiple of 8, so that tile id -> XCD stays id mod 8 as in the tile map.
    const int64_t units = compute_units() / 8 * 8;
    if (units < 8) return hipErrorInvalidValue;
    hipLaunchKernelGGL((k_int8_gemm_persistent<WM, WN, TM, TN, BK, STAGES, OUT>),
                       dim3((unsigned)std::min(total, units)), dim3(64 * WM * WN), lds_bytes, stream,
                       A + pn.row0 * BK, B + pn.col0 * BK, C, Mp, Np, Kp / BK, (int)(k_begin / BK),
                       (int)(k_len / BK), pn.c_ld, pn.c_plane, tm, (int)total, mods);
    return hipGetLastError();
}

template <int WM, int WN, int TM, int TN, int BK, int STAGES, int OUT>
hipError_t launch(const int8_t *A, const int8_t *B, void *C, int batch, int64_t Mp, int64_t Np,
                  int64_t Kp, int64_t k_begin, int64_t k_len, const GemmPanel &pn,
                  const GemmMods &mods, hipStream_t stream) {
    constexpr int BM = 32 * TM * WM, BN = 32 * TN * WN;
    constexpr size_t lds_bytes = (size_t)STAGES * (BM + BN) * BK;
    static thread_local int attr_device = -1;                // the attribute is per device (set again per thread: harmless)
    int dev = -1;
    if (hipError_t e = hipGetDevice(&dev)) return e;
    if (attr_device != dev) {
        hipError_t e = hipFuncSetAttribute(
            reinterpret_cast<const void *>(&k_int8_gemm<WM, WN, TM, TN, BK, STAGES, OUT>),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_device = dev;
    }
    TileMap tm;
    tm.tiles_m = (int)(pn.rows / BM);
    tm.tiles_n = (int)(pn.cols / BN);
    tm.swizzled = (tm.tiles_m % 16 == 0 && tm.tiles_n % 16 == 0) ? 1 : 0;
    const int64_t total = (int64_t)tm.tiles_m * tm.tiles_n * batch;
    if (total > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL((k_int8_gemm<WM, WN, TM, TN, BK, STAGES, OUT>), dim3((unsigned)total),
                       dim3(64 * WM * WN), lds_bytes, stream, A + pn.row0 * BK, B + pn.col0 * BK, C, Mp,
                       Np, Kp / BK, (int)(k_begin / BK), (int)(k_len / BK), pn.c_ld, pn.c_plane, tm, mods);
    return hipGetLastError();
}

template <int OUT>
hipError_t launch_out(const int8_t *A, const int8_t *B, void *C, int batch, int64_t Mp, int64_t Np,
                      int64_t Kp, int64_t k_begin, int64_t k_len, const GemmPanel &pn,
                      const GemmMods &mods, hipStream_t stream) {
    // Problems of fewer than 128 large tiles get the 128 x 128 tile so that more workgroups exist
    // (measured at N = 14: 512^3, 56 large tiles, 11.4 against 17.3 us; 1024^3, 224 large tiles,
    // 31.2 against 26.8 us, so from there on the large tile wins although it leaves units idle).
    if (pn.rows * pn.cols * batch < (int64_t)256 * 256 * 128)
        return launch<2, 2, 2, 2, 64, 4, OUT>(A, B, C, batch, Mp, Np, Kp, k_begin, k_len, pn, mods, stream);
    // 8 wavefronts (2 per SIMD), each 128 x 64: measured against 4 wavefronts of 128 x 128 on
    // the same device it is 2 % faster at 16 x 16384^3 -- a wavefront that is held up issuing
    // a load leaves the matrix core to its SIMD partner.
    if (k_len <= kPersistentMaxK)                      // short contraction: see k_int8_gemm_persistent
        return launch_persistent<2, 4, 4, 2, 64, 4, OUT>(A, B, C, batch, Mp, Np, Kp, k_begin, k_len, pn, mods,
                                                         stream);
    return launch<2, 4, 4, 2, 64, 4, OUT>(A, B, C, batch, Mp, Np, Kp, k_begin, k_len, pn, mods, stream);
}

}  // namespace

hipError_t launch_int8_gemm_maxima(const int8_t *A, const int8_t *B, int64_t Mp, int64_t Np, int64_t Kp,
                                   int64_t k_begin, int64_t k_len, const GemmPanel &pn, int64_t valid_rows,
                                   int64_t valid_cols, int *row_max, int *col_max, hipStream_t stream) {
    if (pn.row0 < 0 || pn.col0 < 0 || pn.rows < kPadMN || pn.cols < kPadMN || pn.row0 % kPadMN ||
        pn.col0 % kPadMN || pn.rows % kPadMN || pn.cols % kPadMN || pn.row0 + pn.rows > Mp ||
        pn.col0 + pn.cols > Np || valid_rows < 0 || valid_cols < 0 || valid_rows > pn.rows ||
        valid_cols > pn.cols || k_begin < 0 || k_len < kPadK || k_len > kMaxExactK || k_begin % kPadK ||
        k_len % kPadK || k_begin + k_len > Kp || !row_max || !col_max)
        return hipErrorInvalidValue;
    // the kernel's view of these arguments: see kOutMax
    GemmPanel q = pn;
    q.c_ld = valid_rows | (valid_cols << 32);
    q.c_plane = col_max - row_max;
    const GemmMods none{};
    if (pn.rows * pn.cols < (int64_t)256 * 256 * 128)        // as in launch_out
        return launch<2, 2, 2, 2, 64, 4, kOutMax>(A, B, row_max, 1, Mp, Np, Kp, k_begin, k_len, q, none, stream);
    return launch<2, 4, 4, 2, 64, 4, kOutMax>(A, B, row_max, 1, Mp, Np, Kp, k_begin, k_len, q, none, stream);
}

hipError_t launch_int8_gemm(const int8_t *A, const int8_t *B, void *C, int batch, int64_t Mp,
                            int64_t Np, int64_t Kp, int64_t k_begin, int64_t k_len, bool as_u8,
                            bool fold, const ModArgs *ma, hipStream_t stream, const GemmPanel *panel) {
    const GemmPanel whole{0, Mp, 0, Np, Np, Mp * Np};
    const GemmPanel &pn = panel ? *panel : whole;
    if (pn.row0 < 0 || pn.col0 < 0 || pn.rows < kPadMN || pn.cols < kPadMN || pn.row0 % kPadMN ||
        pn.col0 % kPadMN || pn.rows % kPadMN || pn.cols % kPadMN || pn.row0 + pn.rows > Mp ||
        pn.col0 + pn.cols > Np || pn.c_ld < pn.cols || pn.c_ld % 16 || pn.c_plane % 16)
        return hipErrorInvalidValue;                       // whole tiles, 16-byte stores
    GemmMods mods{};
    if (ma)
        for (int i = 0; i < ma->n; ++i) { mods.p[i] = ma->p[i]; mods.pinv_prime[i] = (int32_t)ma->pinv_prime[i]; }
    else if (as_u8 || fold)
        return hipErrorInvalidValue;                       // the reduced forms need the moduli
    if (as_u8)
        return fold ? launch_out<kOutU8Fold>(A, B, C, batch, Mp, Np, Kp, k_begin, k_len, pn, mods, stream)
                    : launch_out<kOutU8>(A, B, C, batch, Mp, Np, Kp, k_begin, k_len, pn, mods, stream);
    return fold ? launch_out<kOutI32Fold>(A, B, C, batch, Mp, Np, Kp, k_begin, k_len, pn, mods, stream)
                : launch_out<kOutI32>(A, B, C, batch, Mp, Np, Kp, k_begin, k_len, pn, mods, stream);
}

}  // namespace oz2
