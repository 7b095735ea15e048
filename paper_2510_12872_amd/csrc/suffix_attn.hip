// kvcomm_suffix_attn: causal attention of the non-shared suffix queries over the assembled,
// aligned cache (workflow step 4 of the paper; q, k, v as in Sec. 3.1).  Suffix query i sits
// at cache position n_ctx + i and sees keys 0 .. n_ctx + i.
//
// bf16 path (attn_mfma_kernel): flash-style single pass on bf16 MFMA (32x32x16) with fp32
// accumulation and an fp32 online softmax, written for gfx950:
//   * GQA packing: the G query heads that share a kv head are folded into the row axis of one
//     tile (row r = i * G + g), so each K/V tile staged in LDS serves G heads at once.
//   * Both products are computed transposed, S^T = K Q^T and O^T = V^T P^T.  In the 32x32
//     accumulator layout a lane then owns ONE query column: row max and row sum of the softmax
//     are in-register reductions plus one v_permlane32_swap, the rescale of O is a per-lane
//     scalar, and the exponentiated scores are already laid out as the B operand of the second
//     product (the key order inside a 16-key step is a fixed permutation, matched on the V side).
//   * K and V tiles travel global -> LDS with global_load_lds_dwordx4 (no registers, no LDS
//     stores), issued through inline assembly with a scalar row base and a fixed per-lane offset;
//     the XOR swizzle of 16-byte chunks that keeps operand reads bank-conflict free is
//     applied by choosing which global chunk each lane fetches.  K operands are read with
//     ds_read_b128; V^T operands with ds_read_b64_tr_b16, which transposes on the way out of
//     LDS, so V is never transposed by the vector ALU.
//   * Work advances in 32-key sub-steps as a three-stage software pipeline inside each wavefront:
//     in one step the matrix cores compute S(u+2) = K(u+2) Q^T and O += V(u) P(u), their MFMAs
//     alternating (two independent accumulator chains), while the vector ALU turns S(u+1) into
//     P(u+1).  The vector work is cut into one piece per MFMA and staggered so that no instruction
//     reads what its own piece produced; every piece is pinned by a scheduling barrier.
//   * The softmax reference is not tracked.  It is set from the first sub-step (key 0 is visible to
//     every query) and a sub-step only checks that the row sum of its exponentials, which is needed
//     anyway, stayed below 2^30; a row that did not is re-referenced to its true maximum (O and
//     the running sum rescaled, the exponentials formed again).  Numerator and denominator share
//     the reference, so the result is that of the usual online softmax.  Row sums are plain fp32
//     additions of the unrounded exponentials.
//   * One barrier per 64 keys; K is kept in a ring of four 32-key halves and V in two 64-key
//     tiles so that loads run 1-2 tiles ahead of their use.
//   * A block is eight wavefronts (two per SIMD, 256 registers each) = 256 rows of the packed
//     (query, head) axis = 64 queries of all four heads for G = 4; one block per CU.
//   * Row tiles are ordered longest-first and the block index is remapped so that the row
//     tiles of one (layer, kv head) run on the same XCD and share its L2.
// fp32 path (attn_f32_kernel): one wavefront per query row, plain fp32 FMA and expf with an
// online softmax over 64-key chunks; it exists for exactness, not speed.
#include <math.h>
#include <type_traits>

#include "kvcomm_device.h"

namespace {

using namespace kvc;

struct AttnParams {
    const void *q, *k, *v;
    void *out;
    float *lse;
    Strides s_q, s_k, s_v, s_o;
    int32_t L, Hkv, G, n_ctx, tq, N;
    int32_t n_row_tiles;
    int32_t n_items;   // L * Hkv * n_row_tiles
    float scale;       // softmax scale
    float scale_log2;  // scale * log2(e)
};

// ------------------------------------------------------------------------------- bf16 MFMA
#ifndef KVC_ATTN_WPE
#define KVC_ATTN_WPE 2
#endif
#ifndef KVC_ATTN_NW
#define KVC_ATTN_NW 8  // measured: 2 % faster than two blocks of 4 per CU (every K/V tile enters LDS once per CU)
#endif

__device__ __forceinline__ bf16x8 as_bf16x8(const u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef short s16x4 __attribute__((ext_vector_type(4)));

// Two 8-byte transposing LDS reads (ds_read_b64_tr_b16) -> one 8 x bf16 MFMA operand.
// Within each group of 16 lanes the instruction returns to lane i, element e, the 16-bit
// element (i % 4) found at the address supplied by lane 4*e + i/4 of the group.
__device__ __forceinline__ bf16x8 lds_read_tr_pair(const lds_byte *a0, const lds_byte *a1)
{
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a0);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4 *)a1);
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// One wavefront-wide direct load global -> LDS (global_load_lds_dwordx4): lane i moves the 16 bytes at
// global address `base` + `voff` (a wavefront-uniform 64-bit base in scalar registers plus its own unsigned
// 32-bit byte offset) to LDS address `dst` + 16 * i (`dst` is wavefront-uniform and travels in M0).
// Written as inline assembly on purpose: the compiler then does not know of the pending LDS write and
// inserts no wait of its own before later LDS reads (it would wait for ALL outstanding loads ahead of the
// first transposing read and so serialise the prefetch).  Ordering is explicit instead: tile_barrier()
// waits for the loads (vmcnt) and synchronises the block before anybody reads what they wrote.
// M0 is listed as clobbered, so the compiler re-forms it for any instruction of its own that needs it.
// (clang warns about any reserved register in a clobber list; for M0, which it only ever sets immediately
// before the instruction that reads it, the declaration is exactly what is meant.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16_sbase(const unsigned char *base, uint32_t voff, const lds_byte *dst)
{
    const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)dst);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(base), "s"(m0) : "memory", "m0");
}

template <int V>
using template_int = std::integral_constant<int, V>;

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// The same with the LDS destination as a wavefront-uniform base plus a literal (M0 is formed by one scalar
// add): the steady-state loads then cost no vector ALU instruction and no register per destination (the
// row base advances on the scalar unit and the per-lane offset never changes).
template <int OFF>
__device__ __forceinline__ void dma16_sbase_at(const unsigned char *base, uint32_t voff, uint32_t dst_base)
{
    asm volatile("s_add_u32 m0, %2, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 : : "v"(voff), "s"(base), "s"(dst_base), "n"(OFF) : "memory", "scc", "m0");
}
#pragma clang diagnostic pop

// PERSIST: the grid is smaller than the number of (layer, kv head, row tile) items and every block walks a
// fixed share of them (the items of its XCD, strided by the XCD's number of blocks), so that the kernel occupies
// gridDim.x CUs only and leaves the rest of the chip to whatever runs beside it.  The arithmetic of an item is
// the same instruction sequence as in the one-item-per-block form.
template <int D, int NW, int WPE, bool PERSIST>
__global__ __launch_bounds__(64 * NW, WPE) void attn_mfma_kernel(const AttnParams p_arg)
{
    // PERSIST reads the parameters through an opaque pointer to the kernel-argument segment, once per item:
    // they are then re-loaded (scalar loads) for every item instead of being held in scalar registers for the
    // whole kernel, which the register budget does not allow.
    using ParamT = std::conditional_t<PERSIST, const __attribute__((address_space(4))) AttnParams, const AttnParams>;
    ParamT *p_ptr;
    if constexpr (PERSIST)
        p_ptr = (ParamT *)__builtin_amdgcn_kernarg_segment_ptr();
    else
        p_ptr = &p_arg;
    ParamT &p0 = *p_ptr;
    constexpr int NKS = D / 16;      // k-steps of S^T = K Q^T; also the MFMAs of O^T += V^T P^T per sub-step
    constexpr int NDB = D / 32;      // 32-row blocks of O^T
    constexpr int BM = 32 * NW;      // query rows per block (32 per wavefront)
    constexpr int RW = 64 / NW;      // key rows of a 64-key group that one wavefront loads
    constexpr int KCH = D / 8;       // 16-byte chunks per K / V row
    constexpr int ROWB = D * 2;      // bytes per K / V row
    constexpr int HALFB = 32 * ROWB; // bytes of a 32-key half tile
    constexpr int TILEB = 64 * ROWB; // bytes of a 64-key tile
    constexpr int RPL = 64 / KCH;    // key rows filled by one wavefront-wide direct load
    constexpr int LPT = RW / RPL;    // direct loads per wavefront, tensor and 64-key group
    constexpr int KSWZ = (KCH < 16 ? KCH : 16) - 1; // K chunk swizzle: c ^ (key & KSWZ)
    constexpr int VSWZ = KCH - 1;                   // V chunk swizzle: c ^ ((4 * (key & 3)) & VSWZ)

    // K: ring of four 32-key halves (half h in slot h & 3); V: two 64-key tiles (tile t in buffer t & 1).
    // Rows are [key][D] with XOR-swizzled 16-byte chunks.
    // After the last tile the same memory stages the output rows (32 rows per wavefront) for coalesced stores;
    // the table of row pointers sits behind it.
    __shared__ __align__(16) unsigned char smem[4 * HALFB + 2 * TILEB + NW * 32 * 8];
    static_assert(NW * 32 * ROWB <= 4 * HALFB + 2 * TILEB, "output staging must fit the K / V buffers");
    lds_byte *kring = (lds_byte *)smem;
    lds_byte *vbuf = kring + 4 * HALFB;

    // XCD-aware item order: hardware deals consecutive block ids round-robin to the 8 XCDs; each XCD gets one
    // contiguous range of the items (the row tiles of a (layer, kv head) then share its L2).  Block b is the
    // (b / 8)-th block of XCD b % 8 and takes that range's items b / 8, b / 8 + (blocks of the XCD), ...
    const int x_id = blockIdx.x & 7;
    const int x_first = x_id * (p0.n_items >> 3) + min(x_id, p0.n_items & 7);
    const int x_count = (p0.n_items >> 3) + (x_id < (p0.n_items & 7) ? 1 : 0);
    const int x_blocks = PERSIST ? ((int)gridDim.x - x_id + 7) >> 3 : x_count;
    int item = blockIdx.x >> 3;
    if (PERSIST && item >= x_count) return;   // the whole block: more blocks than items on this XCD
    do {
    int logical = x_first + item;
    int tid = threadIdx.x;
    ParamT *p_item = p_ptr;
    if constexpr (PERSIST) {
        // opaque per item: nothing derived from the item, the thread id or the parameters is kept in registers
        // across items
        asm volatile("" : "+s"(logical));
        asm volatile("" : "+v"(tid));
        asm volatile("" : "+s"(p_item));
    }
    ParamT &p = *p_item;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, n = lane & 31, hg = lane >> 5;
    const int lh = logical / p.n_row_tiles;
    const int rt = p.n_row_tiles - 1 - logical % p.n_row_tiles;  // longest rows first
    const int l = lh / p.Hkv, hkv = lh % p.Hkv;

    const bf16_t *kb_ = static_cast<const bf16_t *>(p.k) + l * p.s_k.layer + hkv * p.s_k.head;
    const bf16_t *vb_ = static_cast<const bf16_t *>(p.v) + l * p.s_v.layer + hkv * p.s_v.head;

    // Every wavefront of the block walks the same tiles (one barrier per 64-key tile); the causal
    // mask is applied from the first 32-key sub-step that is partly hidden from some query of the block.
    const int wg_imax = min(p.tq - 1, (rt * BM + BM - 1) / p.G);
    const int wg_imin = min(p.tq - 1, (rt * BM) / p.G);
    const int n_tiles = (p.n_ctx + wg_imax + 1 + 63) / 64;
    const int n_sub = 2 * n_tiles;
    const int sub_unmasked = (p.n_ctx + wg_imin + 1) / 32;  // sub-steps [0, sub_unmasked) are visible to all queries

    f32x16 o[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int j = 0; j < 16; ++j) o[db][j] = 0.f;

    // ---- global -> LDS direct loads (global_load_lds_dwordx4): lane i of a wavefront fills the
    // 16-byte LDS chunk (base + i); the swizzle is applied by choosing which global chunk it fetches.
    // One instruction fills RPL consecutive key rows.  Addresses are a wavefront-uniform row pointer
    // plus a per-lane byte offset that does not change from tile to tile.
    // In a 64-key group, wavefront w fills keys [RW*w, RW*w + RW); load `it` fills rows RW*w + it*RPL ...
    auto in_row_k = [&](int it) __attribute__((always_inline)) -> int {  // swizzled source chunk (bytes inside the row), K
        const int key = wave * RW + it * RPL + lane / KCH;   // only the row index modulo 16 matters
        return ((lane % KCH) ^ (key & KSWZ)) * 16;
    };
    auto in_row_v = [&](int it) __attribute__((always_inline)) -> int {  // same for V (identical for every `it` when RPL is a multiple of 4)
        const int key = wave * RW + it * RPL + lane / KCH;
        return ((lane % KCH) ^ ((4 * (key & 3)) & VSWZ)) * 16;
    };
    uint32_t ld_koff[LPT], ld_voff[LPT];
#pragma unroll
    for (int it = 0; it < LPT; ++it) {
        ld_koff[it] = (uint32_t)((lane / KCH) * p.s_k.token * 2 + in_row_k(it));
        ld_voff[it] = (uint32_t)((lane / KCH) * p.s_v.token * 2 + in_row_v(it));
    }
    const unsigned char *kbytes = reinterpret_cast<const unsigned char *>(kb_);
    const unsigned char *vbytes = reinterpret_cast<const unsigned char *>(vb_);

    // 64 keys starting at key0 (a multiple of 64) -> K ring; its two halves are h0 = key0/32 and h0+1.
    // A half outside [0, n_sub) is skipped.  The lower NW/2 wavefronts fill the first half, the rest the second.
    // General form (prologue and the last tiles): rows past the cache end re-read the last row; such
    // rows are never unmasked.  The row base is clamped on the scalar unit and a lane whose row would
    // still fall behind the end steps its offset back by whole rows.
    const int lq = lane / KCH;  // this lane's row inside a load
    const uint32_t k_row_bytes = (uint32_t)(p.s_k.token * 2), v_row_bytes = (uint32_t)(p.s_v.token * 2);
    auto load_rows = [&](const unsigned char *bytes, int64_t tok_stride, uint32_t row_bytes, int row0, uint32_t voff,
                         const lds_byte *dst) __attribute__((always_inline)) {
        const int row0c = min(row0, p.N - 1);            // wavefront-uniform
        const int excess = max(lq - (p.N - 1 - row0c), 0);  // rows this lane would overshoot by
        dma16_sbase(bytes + (int64_t)row0c * tok_stride * 2, voff - (uint32_t)excess * row_bytes, dst);
    };
    auto load_k64 = [&](int key0) __attribute__((always_inline)) {
        const int h = key0 / 32 + wave / (NW / 2);
        if (h >= n_sub) return;  // wavefront-uniform
        const int rbase = (wave % (NW / 2)) * RW;
#pragma unroll
        for (int it = 0; it < LPT; ++it)
            load_rows(kbytes, p.s_k.token, k_row_bytes, 32 * h + rbase + it * RPL, ld_koff[it],
                      kring + (h & 3) * HALFB + (rbase + it * RPL) * ROWB);
    };
    auto load_v64 = [&](int tile) __attribute__((always_inline)) {
        if (tile >= n_tiles) return;
#pragma unroll
        for (int it = 0; it < LPT; ++it)
            load_rows(vbytes, p.s_v.token, v_row_bytes, 64 * tile + wave * RW + it * RPL, ld_voff[it],
                      vbuf + (tile & 1) * TILEB + (wave * RW + it * RPL) * ROWB);
    };
    // The first tiles are requested before anything else is set up: their latency is the block's start-up time.
    load_k64(0);    // halves 0, 1
    load_k64(64);   // halves 2, 3
    load_v64(0);
    // This lane's query column: row r = i * G + g of the (layer, kv head) group.
    int qi;
    bf16x8 qf[NKS];
    {
        const int r_row = rt * BM + wave * 32 + n;
        qi = min(r_row / p.G, p.tq - 1);
        const int hq = hkv * p.G + r_row % p.G;
        const bf16_t *qrow = static_cast<const bf16_t *>(p.q) + l * p.s_q.layer + (int64_t)(uint32_t)hq * p.s_q.head + (int64_t)(uint32_t)qi * p.s_q.token;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[ks] = as_bf16x8(load16(qrow + ks * 16 + hg * 8));
    }

    // Steady state (all rows exist, no half is skipped): the same loads from two running row pointers,
    // so that a load costs one 64-bit scalar add instead of a 64-bit multiply, and with M0 formed from
    // a per-wavefront LDS base plus a literal.  kp / vp point at this wavefront's next row to load:
    // during tile t the K halves 2t+4, 2t+5 (keys 64t+128 ...) and V tile t+1.
    const int64_t k_rpl = (int64_t)RPL * p.s_k.token * 2, v_rpl = (int64_t)RPL * p.s_v.token * 2;
    const int64_t k_adv = (int64_t)(64 - LPT * RPL) * p.s_k.token * 2, v_adv = (int64_t)(64 - LPT * RPL) * p.s_v.token * 2;
    const unsigned char *kp = kbytes + (int64_t)(128 + 32 * (wave / (NW / 2)) + (wave % (NW / 2)) * RW) * p.s_k.token * 2;
    const unsigned char *vp = vbytes + (int64_t)(64 + wave * RW) * p.s_v.token * 2;
    const uint32_t lds0 = (uint32_t)(uintptr_t)kring;
    const uint32_t k_rows = lds0 + (wave % (NW / 2)) * RW * ROWB;
    // t even: halves 2t+4, 2t+5 live in slots 0, 1; t odd: in slots 2, 3
    const uint32_t kdst_a = __builtin_amdgcn_readfirstlane(k_rows + (0 + wave / (NW / 2)) * HALFB);
    const uint32_t kdst_b = __builtin_amdgcn_readfirstlane(k_rows + (2 + wave / (NW / 2)) * HALFB);
    const uint32_t vdst = __builtin_amdgcn_readfirstlane(lds0 + 4 * HALFB + wave * RW * ROWB);
    auto load_kv_next = [&](uint32_t kdst, auto vb) __attribute__((always_inline)) {
        constexpr int VB = decltype(vb)::value;  // V buffer, a literal
        static_for<0, LPT>([&](auto it) __attribute__((always_inline)) {
            constexpr int I = decltype(it)::value;
            if (I > 0) kp += k_rpl;
            dma16_sbase_at<I * RPL * ROWB>(kp, ld_koff[I], kdst);
        });
        kp += k_rpl + k_adv;
        static_for<0, LPT>([&](auto it) __attribute__((always_inline)) {
            constexpr int I = decltype(it)::value;
            if (I > 0) vp += v_rpl;
            dma16_sbase_at<VB * TILEB + I * RPL * ROWB>(vp, ld_voff[I], vdst);
        });
        vp += v_rpl + v_adv;
    };

    // ---- per-lane LDS read offsets
    // K operand (rows = keys): lane (n, hg) reads chunk 2*ks + hg of key n of the half.
    int k_off[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) k_off[ks] = n * ROWB + (((2 * ks + hg) ^ (n & KSWZ)) * 16);
    // V^T operand through transposing reads: lane i of a 16-lane group supplies the address of
    // 4 channels [32*db + 16*gi + 4*(i%4), +4) of key 16*ks + 4*hg + i/4 (second read: + 8 keys).
    int v_off[NDB];
    {
        const int i16 = lane & 15, gi = (lane >> 4) & 1;
        const int row = 4 * hg + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < NDB; ++db) {
            const int col = 32 * db + 16 * gi + 4 * (i16 & 3);
            const int pc = (col >> 3) ^ ((4 * (row & 3)) & VSWZ);
            v_off[db] = row * ROWB + pc * 16 + (col & 7) * 2;
        }
    }
    auto read_k = [&](const lds_byte *kl, int ks) __attribute__((always_inline)) -> bf16x8 {
        return as_bf16x8(*(const __attribute__((address_space(3))) u32x4 *)(kl + k_off[ks]));
    };
    auto read_v = [&](const lds_byte *vl, int i) __attribute__((always_inline)) -> bf16x8 {  // i = ks * NDB + db
        const lds_byte *va = vl + (i / NDB) * 16 * ROWB + v_off[i % NDB];
        return lds_read_tr_pair(va, va + 8 * ROWB);
    };

    // ---- softmax state of this lane's query.
    // m is the REFERENCE the exponentials are taken against (raw score units), mc = m * scale * log2(e).  It is
    // a true maximum when it is set, but it is not tracked: a sub-step only checks that its exponentials stayed
    // in range (their row sum, which is needed anyway, below kOverflow) and re-references the row when they did
    // not.  Numerator and denominator share the reference, so the result is that of the usual online softmax;
    // exponentials beyond 1 cost no accuracy in floating point.
    float m = -INFINITY, mc = 0.f, lsum = 0.f;
    f32x16 sbuf[2];   // scores of sub-step u live in sbuf[u & 1]
    u32x4 pbuf[2][2]; // packed bf16 probabilities of sub-step u live in pbuf[u & 1]

    // P = exp2(s * scale * log2(e) - mc) for the 16 scores of this lane, as packed bf16 B operands, and their sum.
    // The work is cut into the 2 * NKS MFMA slots of a pipeline step and staggered so that no instruction reads
    // what its own slot produced: element j is scaled in slot b-2, exponentiated in slot b-1 and
    // summed / packed in slot b = j * NS / 16 (slots -2 and -1 precede the first MFMA).  A wavefront issues in
    // order, so a dependent chain inside one slot would hold back the next MFMA for its whole latency.
    // Lane (n, hg) holds key rows 8*(j/4) + 4*hg + j%4 of the sub-step; `limit` is its last visible key.
    // Row sums are plain fp32 additions of the unrounded exponentials (two chains): v_dot2 on the rounded pairs
    // would agree with the numerator to the last bit, but it shares a pipeline with the MFMAs and costs four
    // times as much next to them; the difference is a relative 2^-9 / sqrt(keys) of the denominator.
    struct ExpState {
        float x[16], e[16], rs_even, rs_odd;
    };
    auto exp_slot = [&](const f32x16 &s, u32x4 (&pk)[2], ExpState &st, int limit, bool masked, int t, int NS)
                        __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int b = j * NS / 16;
            if (b - 2 == t) {
                float v = s[j];
                if (masked) v = 8 * (j >> 2) + 4 * hg + (j & 3) > limit ? -INFINITY : v;
                st.x[j] = __builtin_fmaf(v, p.scale_log2, -mc);
            }
            if (b - 1 == t) st.e[j] = __builtin_amdgcn_exp2f(st.x[j]);
            if (b == t) {
                if (j & 1) {
                    uint32_t pr = pack_bf16x2(st.e[j - 1], st.e[j]);
                    asm volatile("" : "+v"(pr));  // keeps the conversion in this slot (it would sink to its use, a step later)
                    pk[j >> 3][(j & 7) >> 1] = pr;
                    st.rs_odd += st.e[j];
                } else {
                    st.rs_even += st.e[j];
                }
            }
        }
    };
    // A row whose exponentials left the safe range (or the first sub-step, whose reference is still -inf): take
    // the true maximum of the sub-step as the new reference if it is larger, rescale what has been accumulated,
    // and form the exponentials again.  Rare: the reference only ever moves by more than log2(kOverflow).
    auto rereference = [&](const f32x16 &s, u32x4 (&pk)[2], int limit, bool masked) __attribute__((always_inline)) -> float {
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            float v = s[j];
            if (masked) v = 8 * (j >> 2) + 4 * hg + (j & 3) > limit ? -INFINITY : v;
            mx = fmaxf(mx, v);
        }
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        const float m_new = fmaxf(m, mx);
        // m == -inf only in the first sub-step, where key 0 is visible to every query and nothing is accumulated yet
        const float corr = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m - m_new) * p.scale_log2);
        m = m_new;
        mc = m_new * p.scale_log2;
        lsum *= corr;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int j = 0; j < 16; ++j) o[db][j] *= corr;
        ExpState st;
        st.rs_even = st.rs_odd = 0.f;
#pragma unroll
        for (int t = -2; t < 16; ++t) exp_slot(s, pk, st, limit, masked, t, 16);
        return st.rs_even + st.rs_odd;
    };
    constexpr float kOverflow = 1073741824.f;  // 2^30

    // One pipeline step for sub-step u (U4 = u & 3, a literal at every call site, fixes every ring slot and buffer):
    //   matrix cores:  S(u+2) = K(u+2) Q^T  and  O += V(u) P(u), their MFMAs alternating (two independent chains);
    //   vector ALU:    P(u+1) = exp2(S(u+1) - reference), spread evenly over the MFMAs.
    // DO_QK / DO_EXP are false only in the last two sub-steps.  LDS operands are fetched two MFMAs of their own
    // product ahead; every MFMA + vector chunk is pinned by a scheduling barrier.
    auto step = [&](int u, auto u4c, auto do_qk_c, auto do_exp_c, auto masked_c) __attribute__((always_inline)) {
        constexpr int U4 = decltype(u4c)::value;
        constexpr bool DO_QK = decltype(do_qk_c)::value, DO_EXP = decltype(do_exp_c)::value, MASKED = decltype(masked_c)::value;
        f32x16 &s_acc = sbuf[U4 & 1];
        const f32x16 &s_exp = sbuf[(U4 + 1) & 1];
        const lds_byte *kl = kring + ((U4 + 2) & 3) * HALFB;
        const lds_byte *vl = vbuf + ((U4 >> 1) & 1) * TILEB + (U4 & 1) * HALFB;
        const int limit = p.n_ctx + qi - 32 * (u + 1);  // last visible key of S(u+1), relative to its sub-step
        bf16x8 ka[NKS], va[NKS], pf[2];
        pf[0] = as_bf16x8(pbuf[U4 & 1][0]);
        pf[1] = as_bf16x8(pbuf[U4 & 1][1]);
        if (DO_QK) {
            ka[0] = read_k(kl, 0);
            ka[1] = read_k(kl, 1);
        }
        va[0] = read_v(vl, 0);
        va[1] = read_v(vl, 1);
        ExpState st;
        st.rs_even = st.rs_odd = 0.f;
        if (DO_EXP) {
            exp_slot(s_exp, pbuf[(U4 + 1) & 1], st, limit, MASKED, -2, 2 * NKS);
            exp_slot(s_exp, pbuf[(U4 + 1) & 1], st, limit, MASKED, -1, 2 * NKS);
        }
#pragma unroll
        for (int i = 0; i < NKS; ++i) {
            if (DO_QK) {
                if (i == 0) {
                    f32x16 z;
#pragma unroll
                    for (int j = 0; j < 16; ++j) z[j] = 0.f;
                    s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0], qf[0], z, 0, 0, 0);
                } else {
                    s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[i], qf[i], s_acc, 0, 0, 0);
                }
                if (i + 2 < NKS) ka[i + 2] = read_k(kl, i + 2);
            }
            if (DO_EXP) exp_slot(s_exp, pbuf[(U4 + 1) & 1], st, limit, MASKED, 2 * i, 2 * NKS);
            __builtin_amdgcn_sched_barrier(0);
            o[i % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[i], pf[i / NDB], o[i % NDB], 0, 0, 0);
            if (i + 2 < NKS) va[i + 2] = read_v(vl, i + 2);
            if (DO_EXP) exp_slot(s_exp, pbuf[(U4 + 1) & 1], st, limit, MASKED, 2 * i + 1, 2 * NKS);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (DO_EXP) {
            float rs = st.rs_even + st.rs_odd;
            if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(rs < kOverflow)) != 0, 0)) rs = rereference(s_exp, pbuf[(U4 + 1) & 1], limit, MASKED);
            lsum += rs;
        }
    };
    const auto tile_barrier = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wavefront's direct loads have landed in LDS
        __syncthreads();                     // ... and everybody else's; what was read in this tile is free
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    template_int<0> u0; template_int<1> u1; template_int<2> u2; template_int<3> u3;

    // ---- pipeline over tiles.  During tile t the sub-steps 2t and 2t+1 read K halves 2t+2 and 2t+3 and V tile t;
    // the loads issued at its start (K halves 2t+4, 2t+5 into the slots of halves 2t and 2t+1, V tile t+1 into the
    // buffer of tile t-1) only overwrite what tile t-1 finished reading.
    tile_barrier();

    // Prologue: S(0) and S(1); the reference of every query from S(0) (key 0 is visible to all); P(0).
    {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const lds_byte *kl = kring + h * HALFB;
#pragma unroll
            for (int j = 0; j < 16; ++j) sbuf[h][j] = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                sbuf[h] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_k(kl, ks), qf[ks], sbuf[h], 0, 0, 0);
        }
        lsum = rereference(sbuf[0], pbuf[0], p.n_ctx + qi, true);
    }
    // Halves 0 and 1 have no tile before them: every wavefront must have read them before the loads of the
    // first tile (halves 4 and 5 share their slots) are issued.
    __syncthreads();

    const int t_last = n_tiles - 1;
    // Leading tiles whose exponentials need no mask and whose look-ahead loads stay inside the cache: a tile pair
    // starting at t forms the exponentials of sub-steps up to 2t+4 and loads keys up to 64t + 255.
    const int t_safe = p.N >= 256 ? (p.N - 128) / 64 : 0;
    const int t_plain = max(0, min(min((sub_unmasked - 1) >> 1, t_last), t_safe));
    // Two tiles (four sub-steps) per trip so that ring slots and buffers are compile-time constants.
    auto tile_pair = [&](int t, auto plain) __attribute__((always_inline)) {
        constexpr bool PLAIN = decltype(plain)::value;
        using M_ = std::integral_constant<bool, !PLAIN>;
        if (PLAIN) {
            load_kv_next(kdst_a, template_int<1>{});  // K halves 2t+4, 2t+5, V tile t+1
        } else {
            load_k64(64 * t + 128);
            load_v64(t + 1);
        }
        step(2 * t, u0, T_{}, T_{}, M_{});
        step(2 * t + 1, u1, T_{}, T_{}, M_{});
        tile_barrier();
        if (PLAIN) {
            load_kv_next(kdst_b, template_int<0>{});  // K halves 2t+6, 2t+7, V tile t+2
        } else {
            load_k64(64 * t + 192);
            load_v64(t + 2);
        }
        step(2 * t + 2, u2, T_{}, T_{}, M_{});
        step(2 * t + 3, u3, T_{}, T_{}, M_{});
        tile_barrier();
    };
    int t = 0;
    for (; t + 2 <= t_plain; t += 2) tile_pair(t, T_{});
    for (; t + 2 <= t_last; t += 2) tile_pair(t, F_{});
    if (t < t_last) {  // two tiles left (t is even): a whole one, then the last
        load_k64(64 * t + 128);
        load_v64(t + 1);
        step(2 * t, u0, T_{}, T_{}, T_{});
        step(2 * t + 1, u1, T_{}, T_{}, T_{});
        tile_barrier();
        ++t;
        step(2 * t, u2, F_{}, T_{}, T_{});      // S(2t+1) exists already; nothing further to multiply
        step(2 * t + 1, u3, F_{}, F_{}, T_{});  // the last sub-step only adds its V P
    } else {
        step(2 * t, u0, F_{}, T_{}, T_{});
        step(2 * t + 1, u1, F_{}, F_{}, T_{});
    }

    // ---- epilogue: normalise and store; lane (n, hg) holds channels 32*db + 8*(j/4) + 4*hg + j%4 of query row n.
    // Stored straight from these registers a store instruction would scatter 16-byte pieces over 32 rows (8 K
    // partial-line writes per block, several microseconds of back-pressure).  Instead each wavefront passes its
    // 32 rows through LDS (8-byte slots XOR-swizzled with the row number so that neither side conflicts much) and
    // writes them out as whole rows, 16 bytes per lane.
    {
        float ltot;
        {
            const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(lsum), __float_as_uint(lsum), false, false);
            ltot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
        }
        // Row coordinates again, from a freshly read lane id: the compiler then keeps none of the
        // prologue's address terms alive across the tile loops.
        const int lane_e = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        const int n_e = lane_e & 31, hg_e = lane_e >> 5;
        const int r_row = rt * BM + wave * 32 + n_e;
        const bool valid = r_row / p.G < p.tq;
        const uint32_t qi_e = (uint32_t)(r_row / p.G), hq_e = (uint32_t)(hkv * p.G + r_row % p.G);
        bf16_t *orow = static_cast<bf16_t *>(p.out) + l * p.s_o.layer + (int64_t)hq_e * p.s_o.head + (int64_t)qi_e * p.s_o.token;
        constexpr int SLOTS = 2 * KCH;                       // 8-byte slots per row
        constexpr int FM = (SLOTS < 32 ? SLOTS : 32) - 1;    // swizzle mask
        __syncthreads();  // every wavefront has finished reading K and V (and no direct load is outstanding)
        unsigned char *stage = smem + wave * (32 * ROWB);
        uint64_t *ptab = reinterpret_cast<uint64_t *>(smem + 4 * HALFB + 2 * TILEB) + wave * 32;
        if (hg_e == 0) ptab[n_e] = valid ? (uint64_t)(uintptr_t)orow : 0;
        const float inv = 1.f / ltot;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
#pragma unroll
            for (int j4 = 0; j4 < 4; ++j4) {
                u32x2 w;
                w[0] = pack_bf16x2(o[db][4 * j4] * inv, o[db][4 * j4 + 1] * inv);
                w[1] = pack_bf16x2(o[db][4 * j4 + 2] * inv, o[db][4 * j4 + 3] * inv);
                const int slot = (8 * db + 2 * j4 + hg_e) ^ (n_e & FM);
                *reinterpret_cast<u32x2 *>(stage + n_e * ROWB + slot * 8) = w;
            }
        if (p.lse && hg_e == 0 && valid)
            p.lse[((int64_t)l * p.Hkv * p.G + hq_e) * p.tq + qi_e] = m * p.scale + logf(ltot);
        // the reads below touch what other lanes of this wavefront wrote: LDS operations of a wavefront complete in order
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int RPS = 64 / KCH;   // rows per store instruction
        const int c = lane_e % KCH;
#pragma unroll
        for (int it = 0; it < 32 / RPS; ++it) {
            const int row = it * RPS + lane_e / KCH;
            const int f = row & FM;
            const u32x2 lo = *reinterpret_cast<const u32x2 *>(stage + row * ROWB + ((2 * c) ^ f) * 8);
            const u32x2 hi = *reinterpret_cast<const u32x2 *>(stage + row * ROWB + ((2 * c + 1) ^ f) * 8);
            bf16_t *dst = reinterpret_cast<bf16_t *>((uintptr_t)ptab[row]);
            if (dst) {
                const u32x4 v = {lo[0], lo[1], hi[0], hi[1]};
                *reinterpret_cast<u32x4 *>(dst + c * 8) = v;
            }
        }
    }
    if (!PERSIST) break;
    __syncthreads();   // the staging area becomes the K / V buffers of the next item
    item += x_blocks;
    } while (item < x_count);
}

// ------------------------------------------------------------------------------- fp32 path
template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(const AttnParams p)
{
    constexpr int CPL = D / 64;  // output channels per lane
    __shared__ float q_lds[4][D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + wave;  // over (l, hq, i)
    const int Hq = p.Hkv * p.G;
    if (row >= (int64_t)p.L * Hq * p.tq) return;
    const int i = (int)(row % p.tq);
    const int hq = (int)((row / p.tq) % Hq);
    const int l = (int)(row / ((int64_t)p.tq * Hq));
    const int hkv = hq / p.G;
    const float *q = static_cast<const float *>(p.q) + l * p.s_q.layer + (int64_t)hq * p.s_q.head + i * p.s_q.token;
    const float *k = static_cast<const float *>(p.k) + l * p.s_k.layer + (int64_t)hkv * p.s_k.head;
    const float *v = static_cast<const float *>(p.v) + l * p.s_v.layer + (int64_t)hkv * p.s_v.head;
    for (int c = lane; c < D; c += 64) q_lds[wave][c] = q[c];
    // only this wavefront reads q_lds[wave]; its writes are ordered before the reads below
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    const int last = p.n_ctx + i;
    float m = -INFINITY, lsum = 0.f;
    float acc[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = 0.f;

    for (int j0 = 0; j0 <= last; j0 += 64) {
        const int j = j0 + lane;
        float sc = -INFINITY;
        if (j <= last) {
            const float *kr = k + (int64_t)j * p.s_k.token;
            float dot = 0.f;
#pragma unroll 4
            for (int c = 0; c < D; c += 4) {
                const f32x4 kv = *reinterpret_cast<const f32x4 *>(kr + c);
                dot = fmaf(q_lds[wave][c], kv[0], dot);
                dot = fmaf(q_lds[wave][c + 1], kv[1], dot);
                dot = fmaf(q_lds[wave][c + 2], kv[2], dot);
                dot = fmaf(q_lds[wave][c + 3], kv[3], dot);
            }
            sc = dot * p.scale;
        }
        float cmax = sc;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) cmax = fmaxf(cmax, __shfl_xor(cmax, off));
        const float m_new = fmaxf(m, cmax);  // finite: lane 0 of every chunk is visible
        const float corr = expf(m - m_new);
        const float pj = j <= last ? expf(sc - m_new) : 0.f;
        float psum = pj;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) psum += __shfl_xor(psum, off);
        lsum = lsum * corr + psum;
        m = m_new;
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] *= corr;
        const int cnt = min(64, last - j0 + 1);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pv = __shfl(pj, jj);
            const float *vr = v + (int64_t)(j0 + jj) * p.s_v.token;
#pragma unroll
            for (int c = 0; c < CPL; ++c) acc[c] = fmaf(pv, vr[lane + 64 * c], acc[c]);
        }
    }
    float *o = static_cast<float *>(p.out) + l * p.s_o.layer + (int64_t)hq * p.s_o.head + i * p.s_o.token;
    const float inv = 1.f / lsum;
#pragma unroll
    for (int c = 0; c < CPL; ++c) o[lane + 64 * c] = acc[c] * inv;
    if (p.lse && lane == 0) p.lse[row] = m + logf(lsum);
}

}  // namespace

extern "C" size_t kvcomm_suffix_attn_workspace(const kvcomm_model *, int32_t, int32_t) { return 0; }

namespace {

// max_blocks > 0: at most that many thread blocks (the bf16 kernel's persistent form when there are more items).
int suffix_attn(const kvcomm_model *model, kvcomm_tensor q, kvcomm_tensor cache_k, kvcomm_tensor cache_v, int32_t n_ctx,
                int32_t tq, float softmax_scale, kvcomm_tensor out, float *lse_out, int32_t max_blocks, void *stream)
{
    int st = check_model(model);
    if (st) return st;
    if (tq <= 0 || n_ctx < 0) return KVCOMM_EINVAL;
    const int dt = model->dtype;
    if ((st = check_tensor(q, dt, true)) || (st = check_tensor(cache_k, dt, true)) ||
        (st = check_tensor(cache_v, dt, true)) || (st = check_tensor(out, dt, true)))
        return st;

    AttnParams p{};
    p.q = q.ptr;
    p.k = cache_k.ptr;
    p.v = cache_v.ptr;
    p.out = out.ptr;
    p.lse = lse_out;
    p.s_q = strides_of(q);
    p.s_k = strides_of(cache_k);
    p.s_v = strides_of(cache_v);
    p.s_o = strides_of(out);
    p.L = model->n_layers;
    p.Hkv = model->n_kv_heads;
    p.G = model->n_q_heads / model->n_kv_heads;
    p.n_ctx = n_ctx;
    p.tq = tq;
    p.N = n_ctx + tq;
    p.scale = softmax_scale > 0.f ? softmax_scale : (float)(1.0 / sqrt((double)model->head_dim));
    p.scale_log2 = (float)((double)p.scale * 1.4426950408889634);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int D = model->head_dim;

    if (dt == KVCOMM_F32) {
        const int64_t rows = (int64_t)p.L * model->n_q_heads * tq;
        const unsigned n_blocks = (unsigned)((rows + 3) / 4);
        switch (D) {
            case 64: return launch(attn_f32_kernel<64>, dim3(n_blocks), dim3(256), 0, s, p);
            case 128: return launch(attn_f32_kernel<128>, dim3(n_blocks), dim3(256), 0, s, p);
            case 256: return launch(attn_f32_kernel<256>, dim3(n_blocks), dim3(256), 0, s, p);
            default: return KVCOMM_EUNSUPPORTED;
        }
    }

    // The direct loads address a row group as a 64-bit scalar base plus an unsigned 32-bit per-lane byte
    // offset that spans up to 64 * 8 / D rows: the token stride has to leave that offset below 2^32.
    if (D == 64 || D == 128 || D == 256) {
        const int64_t rows_per_load = 64 * 8 / D;
        const int64_t max_tok = ((int64_t)1 << 31) / (2 * rows_per_load);
        if (cache_k.stride_token >= max_tok || cache_v.stride_token >= max_tok) return KVCOMM_EUNSUPPORTED;
    }
    constexpr int NW = KVC_ATTN_NW;    // wavefronts per block
    constexpr int WPE = KVC_ATTN_WPE;  // wavefronts per SIMD the register budget is sized for
    const int bm = D == 256 ? 128 : 32 * NW;
    p.n_row_tiles = (p.G * tq + bm - 1) / bm;
    p.n_items = p.L * p.Hkv * p.n_row_tiles;
    if (max_blocks > 0 && max_blocks < p.n_items) {
        const unsigned n_blocks = (unsigned)max_blocks;
        switch (D) {
            case 64: return launch(attn_mfma_kernel<64, NW, WPE, true>, dim3(n_blocks), dim3(64 * NW), 0, s, p);
            case 128: return launch(attn_mfma_kernel<128, NW, WPE, true>, dim3(n_blocks), dim3(64 * NW), 0, s, p);
            case 256: return launch(attn_mfma_kernel<256, 4, 1, true>, dim3(n_blocks), dim3(256), 0, s, p);
            default: return KVCOMM_EUNSUPPORTED;
        }
    }
    const unsigned n_blocks = (unsigned)p.n_items;
    switch (D) {
        case 64: return launch(attn_mfma_kernel<64, NW, WPE, false>, dim3(n_blocks), dim3(64 * NW), 0, s, p);
        case 128: return launch(attn_mfma_kernel<128, NW, WPE, false>, dim3(n_blocks), dim3(64 * NW), 0, s, p);
        case 256: return launch(attn_mfma_kernel<256, 4, 1, false>, dim3(n_blocks), dim3(256), 0, s, p);
        default: return KVCOMM_EUNSUPPORTED;
    }
}

}  // namespace

extern "C" int kvcomm_suffix_attn(const kvcomm_model *model, kvcomm_tensor q, kvcomm_tensor cache_k,
                                  kvcomm_tensor cache_v, int32_t n_ctx, int32_t tq, float softmax_scale,
                                  kvcomm_tensor out, float *lse_out, void *, size_t, void *stream)
{
    return suffix_attn(model, q, cache_k, cache_v, n_ctx, tq, softmax_scale, out, lse_out, 0, stream);
}

extern "C" int kvcomm_suffix_attn_confined(const kvcomm_model *model, kvcomm_tensor q, kvcomm_tensor cache_k,
                                           kvcomm_tensor cache_v, int32_t n_ctx, int32_t tq, float softmax_scale,
                                           kvcomm_tensor out, float *lse_out, int32_t max_blocks, void *stream)
{
    if (max_blocks < 8) return KVCOMM_EINVAL;   // at least one block on each of the 8 XCDs
    return suffix_attn(model, q, cache_k, cache_v, n_ctx, tq, softmax_scale, out, lse_out, max_blocks, stream);
}
