// Prefill attention over the unified pool: prefill_kernel (causal attention of a chunk of prompt tokens
// against the request's pages, on the matrix cores).
#include "ukv_device.h"

namespace ukv {

// ---------------------------------------------------------------------------------------------
// Prefill phase (section 2.1): the queries of a chunk of prompt tokens attend, causally, to the
// request's cache (their own K/V included; the caller has stored them with the bulk store).
//
// Same matrix-core formulation as the grouped-query decode path (v_mfma_f32_16x16x32_bf16; lane l:
// column j = l%16, k-block q = l/16), with the 16 columns of a product now (query row, query head of the
// group) pairs: a workgroup of four waves owns kPrefillCols = 128 such columns of one (request, kv
// head), each wave NB = 2 blocks of 16.  A wave walks the tokens 0 .. (last position of its columns)
// in tiles of 32:
//   S^T[token][column] = K[token][:] . Q[column][:]        (K rows as left operand, q as right operand)
//   O^T[d][column]    += V^T[d][token] . P^T[token][column]
// The S^T results leave lane (j, q) with the scores of column j for the tokens 4q..4q+3 and
// 16+4q..16+4q+3 of the tile, which is the k-block the second product wants from that lane; V^T
// operands come straight from the row-major V tile by transposing LDS reads.  The weights P enter the
// second product in one of two forms (template parameter PARTS):
//   2: split into bf16 high and low parts (two products against the pool's bf16 V rows): 16 mantissa bits;
//   1: rounded to fp16 (one product, v_mfma_f32_16x16x32_f16), 11 significant bits: every weight is off by at most
//      2^-11 of itself, the same rounded weights are summed for the denominator, so a result moves by at most
//      2^-10 times the largest distance of a V element from that result (and by far less unless the rounding
//      errors line up with the V elements).  The matrix instruction wants both
//      operands in one format, so the V rows are read as fp16 from a copy that v16_kernel has made in the
//      workspace (bf16's 8 significant bits fit fp16; values beyond +-65504 saturate, below 2^-24 vanish).
//      The exponentials are taken 2^8 higher, which keeps small weights out of fp16's subnormal range.
// Column j of a block is
// row r0 + blk*(16/G) + j/G, head j%G; the score of (token t, column) counts if t <= position(column)
// -- only the last tiles of a block are partly masked, tiles wholly behind a block's rows are
// skipped.  The tiles are pipelined: while the vector units do the softmax of one tile, the matrix
// cores take the raw scores of the next.  The running maximum starts at a large finite negative
// number, so that a column none of whose tokens has been seen yet stays at weight 0 without inf - inf.
static constexpr float kMinusBig = -1.0e30f;
static constexpr float kLazy = 6.0f; // log2 of the largest weight tolerated before the reference moves
static constexpr float kShiftOnePart = 8.0f; // one-part weights are 2^8 x the two-part ones: at most 2^14, fp16 holds 2^15
// Staged tiles in LDS: the 32 K rows of a tile in one stretch, its 32 V rows in another, 2 head_dim bytes
// per row, written by global-to-LDS loads (no registers in between; lane L of a wave instruction fills
// bytes [16 L, 16 L + 16) of a 1 KiB stretch, from any global address).  Rows keep their 16-byte pieces
// at exclusive-or'ed positions (K: piece ^ (token % pieces); V: see vswz), so that the operand reads of
// adjacent lanes fall on different banks.  Two arrays each for K and V, of two tiles each: one is read
// while the other is written, and the workgroup meets once per pair of tiles (at one tile per array and
// a barrier per tile the kernel was 1.6 % slower on 13 k-token prompts and 2.7 % on the chat mix).
static constexpr int kPfTabWindow = 1024;
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef const __attribute__((address_space(1))) void *global_ptr_t;

template <int NB, int NW, int D, int PARTS>
__global__ void __launch_bounds__(64 * NW, 2) prefill_kernel(PrefillArgs a) {
    // a checked call (UKV_PARAM_VALIDATE) whose page tables hold an id outside the pool does nothing
    if (a.bad != nullptr && uni(*reinterpret_cast<const volatile uint32_t *>(a.bad)) != 0)
        return;
    constexpr int NT = 64 * NW;             // NW = 4 or 8 waves; D = 128 or 64
    constexpr uint32_t KB = 2 * D;          // bytes of the K (or V) part of a head-row
    constexpr uint32_t PIECES = KB / 16;    // 16-byte pieces of it
    constexpr int KSTEPS = D / 32;          // products of 32 along head_dim for one score tile
    constexpr int MM = D / 16;              // products of 16 output rows (head_dim elements) for O^T
    constexpr uint32_t RPI = 1024 / KB;     // head-rows one staging instruction (1 KiB) covers
    constexpr uint32_t KI = 32 / RPI / NW;  // staging instructions per wave, tile and part (K, V)
    static_assert(KI >= 1, "too many waves for this head_dim");
    constexpr uint32_t kPartBytes = 32 * KB; // the K rows (or the V rows) of a 32-token tile
    constexpr float kShift = PARTS == 2 ? 0.f : kShiftOnePart;
    __shared__ PrefillRec s_rec;
    // Two pairs of staged tiles, one array each: with distinct arrays the compiler can tell that reading one pair
    // does not depend on the global-to-LDS loads that fill the other, and lets those loads stay in flight.
    __shared__ __align__(16) unsigned char s_k0[2 * kPartBytes], s_k1[2 * kPartBytes];
    __shared__ __align__(16) unsigned char s_v0[2 * kPartBytes], s_v1[2 * kPartBytes];
    __shared__ int32_t s_ptab[kPfTabWindow]; // page-table window (smaller than the decode path's: the LDS of
                                             // a workgroup sets how many of them fit a CU)
    if (threadIdx.x == 0)
        s_rec = a.recs[blockIdx.x];
    __syncthreads();
    const uint32_t q_len = uni(s_rec.q_len);
    if (q_len == 0)
        return; // filler
    const uint64_t table_off = uni(s_rec.table_off), q_off = uni(s_rec.q_off), out_off = uni(s_rec.out_off);
    const uint32_t ctx_len = uni(s_rec.ctx_len), kvh = uni(s_rec.kvh), r0 = uni(s_rec.r0);
    const unsigned char *v16 = PARTS == 1 ? a.v16 + uni(s_rec.v16_off) : nullptr; // this (request, kv head)'s V rows as fp16
    // G query heads share the kv head; a query row takes GL columns of a block (G rounded up to a power of two)
    const uint32_t G = uni(s_rec.g) & 0xffffu, GL = uni(s_rec.g) >> 16, n_q = uni(s_rec.n_q);
    const uint64_t T = uni(s_rec.token_bytes);
    const float scale_log2e = uni(s_rec.scale_log2e);
    int32_t *tab = s_ptab;

    const int tid = threadIdx.x, lane = tid & 63;
    const uint32_t wave = uni((uint32_t)(tid >> 6));
    const uint32_t j = lane & 15, q = lane >> 4;
    const uint32_t lg = a.log2_page;
    const uint64_t page_mask = (1ull << lg) - 1;
    // this lane's share of a staged tile: piece position lane % PIECES of tokens RPI (KI wave + x) + lane / PIECES
    const uint32_t ld_tok = RPI * KI * wave + lane / PIECES, ld_pos = lane % PIECES;
    // V rows keep their 16-byte pieces at piece ^ vswz(token), which spreads the 32-byte stretches that one
    // transposing read takes from 8 different rows over all banks.  Such a read hands lane i of a group of
    // 16 the element i%4 of what the lanes 4x + i/4 (x = 0..3) of the group addressed: with lane s pointing
    // at elements 16 mm + 4 (s%4) .. +3 of token 4q + s/4, lane i receives V[4q + x][16 mm + i], x = 0..3.
    auto vswz = [](uint32_t tok) { return 2 * ((tok / (256 / KB)) % (KB / 32)); };
    // where, inside a head-row (K) or a row of the fp16 copy (V), the pieces lie that this lane's loads fetch
    uint32_t k_piece[KI], v_piece[KI], kv_delta[KI];
#pragma unroll
    for (uint32_t x = 0; x < KI; ++x) {
        const uint32_t tok = ld_tok + RPI * x;
        k_piece[x] = (ld_pos ^ (tok % PIECES)) * 16;
        v_piece[x] = (ld_pos ^ vswz(tok)) * 16;
        kv_delta[x] = KB + v_piece[x] - k_piece[x]; // from the lane's K piece to its V piece of the same head-row
    }
    uint32_t voff[MM]; // this lane's read offsets into a staged V tile, one per group of 16 output rows
    {
        const uint32_t tok = 4 * q + j / 4, h = j % 4;
#pragma unroll
        for (int mm = 0; mm < MM; ++mm)
            voff[mm] = tok * KB + (((2 * mm + h / 2) ^ vswz(tok)) * 16) + (h % 2) * 8;
    }
    auto vt_operand = [&](const unsigned char *p) { // the tile's tokens 4q..4q+3 from p, tokens 16+4q..16+4q+3 from 16 rows further
        typedef __attribute__((address_space(3))) s16x4_t *lds_s16x4_ptr;
        struct {
            s16x4_t lo, hi;
        } w;
        w.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
        w.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p + 16 * KB));
        return __builtin_bit_cast(uint4, w);
    };
    const uint32_t rpb = 16 / GL;                  // query rows per block of 16 columns
    const uint32_t pos0 = ctx_len - q_len;         // position of query row 0
    const uint32_t row_w = r0 + wave * NB * rpb;   // first row of this wave

    // per block: this lane's column (row, head), its position, and the q operand
    uint32_t col_pos[NB];
    bool col_ok[NB];
    bf16x8_t qreg[NB][KSTEPS]; // the q operands stay in registers: re-reading them from LDS for every tile cost 3 %
    f32x4_t oacc[NB][MM];
    float m[NB], m_lazy[NB]; // reference point of the exponentials, and the maximum above which it moves (m + kLazy)
    f32x4_t lacc[NB]; // running sums of the weights, every element the same (see pv)
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const uint32_t row = row_w + b * rpb + j / GL;
        col_ok[b] = row < q_len && j % GL < G;
        col_pos[b] = pos0 + row;
        const uint4 *qp = reinterpret_cast<const uint4 *>(a.q + q_off + ((uint64_t)(col_ok[b] ? row : 0) * n_q + kvh * G +
                                                                         (col_ok[b] ? j % GL : 0)) * D) + q;
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st) {
            uint4 w = ld_g16(qp + st * 4);
            if (!col_ok[b])
                w = make_uint4(0, 0, 0, 0);
            qreg[b][st] = as_bf16x8(w);
        }
#pragma unroll
        for (int mm = 0; mm < MM; ++mm)
            oacc[b][mm] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
        m[b] = kMinusBig;
        m_lazy[b] = kMinusBig + kLazy;
        lacc[b] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
    }
    // tokens this wave / this workgroup has to look at: up to the position of the last valid row
    auto hi_of = [&](uint32_t first_row, uint32_t n_rows) -> uint32_t {
        if (first_row >= q_len)
            return 0;
        const uint32_t last_row = min(first_row + n_rows, q_len) - 1;
        return pos0 + last_row + 1;
    };
    // ... cut to the stretch [t0, t1) this workgroup was given (the whole of it unless the tile's walk was split)
    const uint32_t t0 = uni(s_rec.t0), t1 = uni(s_rec.t1), part = uni(s_rec.part);
    const uint32_t wave_hi = min(hi_of(row_w, NB * rpb), t1);
    const uint32_t wg_hi = min(hi_of(r0, NW * NB * rpb), t1);
    const uint32_t wave_lo = pos0 + row_w;                     // position of the wave's first row
    const bool wave_full = row_w + NB * rpb <= q_len;          // all the wave's columns are valid rows

    const uint64_t row_off = (uint64_t)kvh * (4 * D);
    uint32_t w0 = t0;
    while (w0 < wg_hi) { // workgroup-uniform: one pass per page-table window
        const uint64_t s_lo = ((uint64_t)w0 * T + row_off) >> lg;
        const uint64_t lim = (s_lo + kPfTabWindow) << lg;
        const uint64_t tmax = (lim - (row_off + 4 * D)) / T; // last token whose head-row ends inside the window
        const uint32_t w1 = (uint32_t)(tmax + 1 < (uint64_t)wg_hi ? tmax + 1 : (uint64_t)wg_hi);
        const uint32_t n_ent = (uint32_t)((((uint64_t)(w1 - 1) * T + row_off + 4 * D - 1) >> lg) - s_lo) + 1;
        if (w0 != 0)
            __syncthreads();
        for (uint32_t e = tid; e < n_ent; e += NT)
            tab[e] = as_global(a.page_table)[table_off + s_lo + e];
        __syncthreads();

        const uint32_t r1 = min(w1, wave_hi); // this wave's tokens of the window end here
        {
            const uint32_t last = w1 - 1;
            // Window-relative byte offsets fit 32 bits (a window spans at most kPfTabWindow pages).
            const uint32_t c0 = (uint32_t)(((uint64_t)w0 * T + row_off) - (s_lo << lg));
            const uint32_t T32 = (uint32_t)T, mask32 = (uint32_t)page_mask;
            // Address of token t's head-row, `add` bytes into it.  The offset inside the window is a product of
            // 24-bit factors (a window holds fewer than 2^24 tokens, a token row is shorter than 2^24 bytes: the
            // full-rate multiply); what is added to the page's address is formed in 32 bits first.
            auto row_ptr = [&](uint32_t t, uint32_t add) -> const unsigned char * {
                const uint32_t off = __umul24(t - w0, T32) + c0;
                const int32_t pg = tab[off >> lg];
                return a.pool_base + (((uint64_t)(uint32_t)pg << lg) + ((off & mask32) + add));
            };
            // Tile staging: each wave fetches RPI KI of the tile's 32 K rows (or V rows), RPI rows per
            // global-to-LDS load.  Tokens past the window's end are copies of its last token (masked in the
            // scores).  A tile's K is requested one step before its V, so the row addresses are worked out
            // once, for K, and kept for V.
            struct RowPtrs { // of this lane's K pieces of a tile (its V pieces: kv_delta[x] further, two-part weights only)
                const unsigned char *p[KI];
            };
            auto rows_of = [&](uint32_t tb) {
                RowPtrs r;
#pragma unroll
                for (uint32_t x = 0; x < KI; ++x)
                    r.p[x] = row_ptr(min(tb + ld_tok + RPI * x, last), k_piece[x]);
                return r;
            };
            auto issue_k = [&](const RowPtrs &r, unsigned char *kt) {
#pragma unroll
                for (uint32_t x = 0; x < KI; ++x)
                    __builtin_amdgcn_global_load_lds((global_ptr_t)(r.p[x]), (lds_ptr_t)(kt + (KI * wave + x) * 1024), 16, 0, 0);
            };
            // V rows of the tile at tb: from the pool (r: the row addresses worked out for the tile's K), or, with
            // one-part weights, from the fp16 copy, whose rows of one kv head follow each other.
            auto issue_v = [&](const RowPtrs &r, uint32_t tb, unsigned char *vt) {
#pragma unroll
                for (uint32_t x = 0; x < KI; ++x) {
                    const unsigned char *src = PARTS == 1 ? v16 + ((uint64_t)min(tb + ld_tok + RPI * x, last) * KB + v_piece[x])
                                                          : r.p[x] + kv_delta[x];
                    __builtin_amdgcn_global_load_lds((global_ptr_t)(src), (lds_ptr_t)(vt + (KI * wave + x) * 1024), 16, 0, 0);
                }
            };
            // Raw scores S^T = K Q^T of one staged K tile against all NB blocks of the wave.
            auto scores = [&](const unsigned char *kt, f32x4_t (&s0)[NB], f32x4_t (&s1)[NB]) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    s0[b] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
                    s1[b] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int st = 0; st < KSTEPS; ++st) { // K rows of tokens j and 16+j, pieces st*4+q
                    const uint32_t pc = ((st * 4 + q) ^ (j % PIECES)) * 16; // (16 + j) % PIECES == j % PIECES
                    const u32x4 k0 = *reinterpret_cast<const u32x4 *>(kt + j * KB + pc);
                    const u32x4 k1 = *reinterpret_cast<const u32x4 *>(kt + (16 + j) * KB + pc);
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const bf16x8_t qb = qreg[b][st];
                        s0[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(k0), qb, s0[b], 0, 0, 0);
                        s1[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(k1), qb, s1[b], 0, 0, 0);
                    }
                }
            };
            // Online softmax of the tile at tb from its raw scores, stage by stage over the blocks, so
            // that the blocks' independent instruction chains can overlap.  MASKED: the tile reaches past
            // some column's position (or past the window); otherwise every score counts and the compares
            // are skipped.  A block that lies wholly before the tile just sees every score masked.
            // Returns whether some accumulator has to be rescaled before the tile is added: by 2^(m_old[b] - m[b]).
            auto softmax = [&](uint32_t tb, const f32x4_t (&s0)[NB], const f32x4_t (&s1)[NB], uint4 (&Ph)[NB],
                               uint4 (&Pl)[NB], float (&m_old)[NB], auto masked) -> bool {
                constexpr bool MASKED = decltype(masked)::value;
                // Raw scores; the scale (times log2 e, positive) is applied to the maximum and folded into
                // the multiply-add under the exponential.
                float sr[NB][8], mt[NB];
#pragma unroll
                for (int b = 0; b < NB; ++b) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        sr[b][r] = s0[b][r];
                        sr[b][4 + r] = s1[b][r];
                    }
                    if (MASKED) {
                        // causal mask: token t counts for this column if t <= its position (and lies in
                        // this window: tokens past it were loaded as copies of the window's last token)
                        const uint32_t t_lim = col_ok[b] ? min(col_pos[b] + 1, r1) : 0;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            sr[b][r] = (tb + 4 * q + r < t_lim) ? sr[b][r] : -INFINITY;
                            sr[b][4 + r] = (tb + 16 + 4 * q + r < t_lim) ? sr[b][4 + r] : -INFINITY;
                        }
                    }
                    mt[b] = fmaxf(fmaxf(fmaxf(sr[b][0], sr[b][1]), fmaxf(sr[b][2], sr[b][3])),
                                  fmaxf(fmaxf(sr[b][4], sr[b][5]), fmaxf(sr[b][6], sr[b][7])));
                }
                max_over_kblocks_pair(mt);
                uint64_t rescale = 0; // lanes one of whose columns moves its reference (kept as a mask: no round trip through a register)
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    // The reference point of the exponentials only moves when the maximum has grown by
                    // more than 2^kLazy: weights then stay below 2^kLazy, and the accumulators are rescaled
                    // rarely (by 2^-grow, worked out only then: see step).
                    mt[b] *= scale_log2e;
                    const bool moves = mt[b] > m_lazy[b];
                    const float mn = moves ? mt[b] : m[b]; // finite: m starts at kMinusBig
                    rescale |= __builtin_amdgcn_ballot_w64(moves);
                    m_old[b] = m[b];
                    m[b] = mn;
                    uint32_t ph[4], pl[4] = {0, 0, 0, 0};
                    const float neg_ref = kShift - mn;
#pragma unroll
                    for (int e = 0; e < 8; e += 2) {
                        const float p0 = fast_exp2(fmaf(sr[b][e], scale_log2e, neg_ref));
                        const float p1 = fast_exp2(fmaf(sr[b][e + 1], scale_log2e, neg_ref));
                        if constexpr (PARTS == 2) {
                            // P as two bf16 parts by truncation (see process_item_gqa)
                            const uint32_t u0 = __float_as_uint(p0), u1 = __float_as_uint(p1);
                            const float x0 = p0 - __uint_as_float(u0 & 0xffff0000u);
                            const float x1 = p1 - __uint_as_float(u1 & 0xffff0000u);
                            ph[e / 2] = __builtin_amdgcn_perm(u1, u0, 0x07060302u);
                            pl[e / 2] = __builtin_amdgcn_perm(__float_as_uint(x1), __float_as_uint(x0), 0x07060302u);
                        } else {
                            ph[e / 2] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{p0, p1}, f16x2_t));
                        }
                    }
                    Ph[b] = make_uint4(ph[0], ph[1], ph[2], ph[3]);
                    Pl[b] = make_uint4(pl[0], pl[1], pl[2], pl[3]);
                }
                return rescale != 0;
            };
            // O^T += V^T P^T for one staged V tile, one group of 16 output rows at a time, multiplied into every
            // block.  The weights' running sums ride along as one more product with an all-ones left operand: every row
            // of its result is the column sum of the (two-part) weights, over all four k-blocks at once.
            auto pv = [&](const unsigned char *vt, const uint4 (&Ph)[NB], const uint4 (&Pl)[NB]) {
                constexpr uint32_t kOne = PARTS == 2 ? 0x3f803f80u : 0x3c003c00u; // 1.0 twice, bf16 or fp16
                const uint4 ones = make_uint4(kOne, kOne, kOne, kOne);
                auto mac = [](const uint4 &x, const uint4 &y, const f32x4_t &c) {
                    if constexpr (PARTS == 2)
                        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(x), as_bf16x8(y), c, 0, 0, 0);
                    else
                        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, x),
                                                                      __builtin_bit_cast(f16x8_t, y), c, 0, 0, 0);
                };
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    lacc[b] = mac(ones, Ph[b], lacc[b]);
                    if constexpr (PARTS == 2)
                        lacc[b] = mac(ones, Pl[b], lacc[b]);
                }
                // Left operand of the product for output rows d = 16 mm + i (lane i of 16): V[token][d] for the
                // lane's 8 tokens, fetched by two transposing LDS reads (tokens 4q..4q+3 and 16+4q..16+4q+3).
                // The reads run two groups ahead of the products that use them (the order is pinned below):
                // issued only when needed, every group of products would wait out a whole LDS round trip.
                uint4 Vt[MM];
#pragma unroll
                for (int mm = 0; mm < MM; ++mm)
                    Vt[mm] = vt_operand(vt + voff[mm]);
#pragma unroll
                for (int mm = 0; mm < MM; ++mm) {
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        oacc[b][mm] = mac(Vt[mm], Ph[b], oacc[b][mm]);
                        if constexpr (PARTS == 2)
                            oacc[b][mm] = mac(Vt[mm], Pl[b], oacc[b][mm]);
                    }
                }
                constexpr int kAhead = 2; // groups of 16 output rows whose operands are in flight
                __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0); // LDS reads of the first groups
                __builtin_amdgcn_sched_group_barrier(0x008, PARTS * NB, 0); // the sums of the weights
#pragma unroll
                for (int mm = 0; mm < MM; ++mm) {
                    if (mm + kAhead < MM)
                        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, PARTS * NB, 0);
                }
            };
            RowPtrs rows; // row addresses of the last tile whose K has been requested (its V is requested a pair later)
            // One tile of the pipeline.  On entry the raw scores of the tile at tb are in c0s/c1s, K of the next tile
            // lies at k_next and V of this tile at v_cur.  The matrix cores take the next tile's scores while the
            // vector units do this tile's softmax -- the two are independent, which is the point of the arrangement --
            // and then this tile's V^T P^T is added.  A wave past its own rows (tb >= r1) does nothing.
            auto tile = [&](uint32_t tb, const unsigned char *k_next, const unsigned char *v_cur, const f32x4_t (&c0s)[NB],
                            const f32x4_t (&c1s)[NB], f32x4_t (&n0s)[NB], f32x4_t (&n1s)[NB]) {
                if (tb < r1) {
                    uint4 Ph[NB], Pl[NB];
                    float m_old[NB];
                    bool rescale;
                    // The next tile's scores are taken whether or not this wave (or the window) has a next
                    // tile: without one they are computed from stale LDS contents and never used.
                    // (Inside either branch, so that the two share a basic block and get interleaved.)
                    // wave-uniform: all 32 tokens lie in the window and at or before the wave's first row,
                    // and every column of the wave is a valid row
                    if (tb + 32 <= r1 && tb + 32 <= wave_lo + 1 && wave_full) {
                        scores(k_next, n0s, n1s);
                        rescale = softmax(tb, c0s, c1s, Ph, Pl, m_old, std::false_type{});
                    } else {
                        scores(k_next, n0s, n1s);
                        rescale = softmax(tb, c0s, c1s, Ph, Pl, m_old, std::true_type{});
                    }
                    if (rescale) {
#pragma unroll
                        for (int b = 0; b < NB; ++b) {
                            const float alpha = fast_exp2(m_old[b] - m[b]); // 1 for a column whose reference stayed
                            m_lazy[b] = m[b] + kLazy;
                            lacc[b] *= alpha;
#pragma unroll
                            for (int mm = 0; mm < MM; ++mm)
                                oacc[b][mm] *= alpha;
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0); // keeps the V registers from being loaded before the scores are done with theirs
                    // A wave that is in its softmax goes first at the instruction issue; one that is in the
                    // run of matrix instructions below needs an issue slot only now and then.  Two waves of a
                    // SIMD then tend to be in different phases, so that vector and matrix units both have work.
                    __builtin_amdgcn_s_setprio(0);
                    pv(v_cur, Ph, Pl);
                    __builtin_amdgcn_s_setprio(2);
                }
            };
            // A pair of tiles between two barriers.  The staging arrays hold two tiles each.  On entry: the scores of
            // the tile at tb are in sa; k_cur holds K of the tiles at tb + 32 and tb + 64, v_cur V of those at tb and
            // tb + 32; `rows` are the row addresses of the tile at tb + 64.  The pair first requests what the next one
            // needs -- K of tb + 96 and tb + 128 into k_fill, V of tb + 64 and tb + 96 into v_fill, the arrays the
            // previous pair has left -- and then works through its two tiles, so that the loads have two tiles' time
            // to arrive and the workgroup meets once per 64 tokens.  Control flow is workgroup-uniform up to the barrier.
            auto pair = [&](uint32_t tb, const unsigned char *k_cur, const unsigned char *v_cur, unsigned char *k_fill,
                            unsigned char *v_fill, f32x4_t (&sa0)[NB], f32x4_t (&sa1)[NB], f32x4_t (&sb0)[NB],
                            f32x4_t (&sb1)[NB]) {
                if (tb + 64 < w1)
                    issue_v(rows, tb + 64, v_fill);
                if (tb + 96 < w1) {
                    rows = rows_of(tb + 96);
                    issue_k(rows, k_fill);
                    issue_v(rows, tb + 96, v_fill + kPartBytes);
                }
                if (tb + 128 < w1) {
                    rows = rows_of(tb + 128);
                    issue_k(rows, k_fill + kPartBytes);
                }
                tile(tb, k_cur, v_cur, sa0, sa1, sb0, sb1);
                if (tb + 32 < w1)
                    tile(tb + 32, k_cur + kPartBytes, v_cur + kPartBytes, sb0, sb1, sa0, sa1);
                __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0): this wave's part of the tiles just requested is in LDS
                __syncthreads(); // they are complete; the arrays just read may be overwritten
            };
            f32x4_t sa0[NB], sa1[NB], sb0[NB], sb1[NB];
            // The window's first tiles: K of the first one into the array the first pair fills (it is read before
            // that), K of the second and third and V of the first two where the first pair expects them.
            rows = rows_of(w0);
            issue_k(rows, s_k1);
            issue_v(rows, w0, s_v0);
            if (w0 + 32 < w1) {
                rows = rows_of(w0 + 32);
                issue_k(rows, s_k0);
                issue_v(rows, w0 + 32, s_v0 + kPartBytes);
            }
            if (w0 + 64 < w1) {
                rows = rows_of(w0 + 64);
                issue_k(rows, s_k0 + kPartBytes);
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads(); // they are staged
            if (w0 < r1)
                scores(s_k1, sa0, sa1);
            __syncthreads(); // every wave is done with the first tile's K
            for (uint32_t tb = w0; tb < w1; tb += 128) { // workgroup-uniform; pairs alternate between the arrays
                pair(tb, s_k0, s_v0, s_k1, s_v1, sa0, sa1, sb0, sb1);
                if (tb + 64 < w1)
                    pair(tb + 64, s_k1, s_v1, s_k0, s_v0, sa0, sa1, sb0, sb1);
            }
        }
        w0 = w1;
    }

    // lane (j, q) holds O[column j][d = 16 mm + 4q + r] in oacc[b][mm][r] and the column's sum of weights in lacc[b]
    if (part != kPrefillDirect) { // one stretch of the tile's tokens: accumulators, reference point and sum as they are
        float *pb = a.partials + (uint64_t)part * kPrefillPartFloats;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (!col_ok[b])
                continue;
            const uint32_t col = (wave * NB + b) * 16 + j;
            float *dst = pb + col * D + 4 * q;
#pragma unroll
            for (int mm = 0; mm < MM; ++mm)
                st_g16(dst + 16 * mm, oacc[b][mm][0], oacc[b][mm][1], oacc[b][mm][2], oacc[b][mm][3]);
            if (q == 0)
                st_g8(pb + kPrefillCols * D + col * 2, m[b], lacc[b][0]);
        }
        return;
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const float lb = lacc[b][0];
        if (!col_ok[b])
            continue;
        const float inv = lb > 0.f ? 1.f / lb : 0.f;
        const uint32_t row = col_pos[b] - pos0;
        float *dst = a.out + out_off + ((uint64_t)row * n_q + kvh * G + j % GL) * D + 4 * q;
#pragma unroll
        for (int mm = 0; mm < MM; ++mm)
            st_g16(dst + 16 * mm, oacc[b][mm][0] * inv, oacc[b][mm][1] * inv, oacc[b][mm][2] * inv,
                   oacc[b][mm][3] * inv);
    }
}

// Merge of the partials of a tile of query rows whose tokens were walked in stretches by several workgroups:
//   out = sum_c O_c 2^(m_c - M) / sum_c l_c 2^(m_c - M),  M = max_c m_c
// (a stretch that lies past a column's position left that column at (m, l) = (very negative, 0): weight 0).
// One workgroup per (tile, block of 16 columns); a thread takes four head_dim elements of one column: first the
// largest reference point over the parts (the (m, l) pairs are few and stay in cache), then the weighted sums, with the
// accumulator loads of four parts in flight.
__global__ void __launch_bounds__(256) prefill_merge_kernel(const PrefillMergeRec *recs, const float *partials,
                                                            float *out, const uint32_t *bad) {
    if (bad != nullptr && uni(*reinterpret_cast<const volatile uint32_t *>(bad)) != 0)
        return;
    const PrefillMergeRec r = recs[blockIdx.x];
    const uint32_t D = r.d, G = r.g & 0xffffu, GL = r.g >> 16, rpb = 16 / GL;
    const uint32_t d4 = D / 4;
    const float *base = partials + (uint64_t)r.part0 * kPrefillPartFloats;
    for (uint32_t u = threadIdx.x; u < 16 * d4; u += 256) {
        const uint32_t j = u / d4, e = (u % d4) * 4, col = blockIdx.y * 16 + j;
        const uint32_t row = r.r0 + blockIdx.y * rpb + j / GL, head = j % GL;
        if (row >= r.q_len || head >= G)
            continue;
        const float *ml = base + kPrefillCols * D + col * 2;
        float M = kMinusBig;
        for (uint32_t c = 0; c < r.n_parts; ++c)
            M = fmaxf(M, ml[(uint64_t)c * kPrefillPartFloats]);
        float L = 0.f, o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f;
        const float *acc = base + col * D + e;
        for (uint32_t c0 = 0; c0 < r.n_parts; c0 += 4) {
            uint4 x[4];
            float w[4], lc[4];
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                const uint32_t c = min(c0 + k, r.n_parts - 1);
                x[k] = ld_g16(acc + (uint64_t)c * kPrefillPartFloats);
                const float mc = ml[(uint64_t)c * kPrefillPartFloats];
                lc[k] = ml[(uint64_t)c * kPrefillPartFloats + 1];
                w[k] = c0 + k < r.n_parts ? fast_exp2(mc - M) : 0.f;
            }
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                L = fmaf(lc[k], w[k], L);
                o0 = fmaf(__uint_as_float(x[k].x), w[k], o0);
                o1 = fmaf(__uint_as_float(x[k].y), w[k], o1);
                o2 = fmaf(__uint_as_float(x[k].z), w[k], o2);
                o3 = fmaf(__uint_as_float(x[k].w), w[k], o3);
            }
        }
        const float inv = L > 0.f ? 1.f / L : 0.f;
        st_g16(out + r.out_off + ((uint64_t)row * r.n_q + r.kvh * G + head) * D + e, o0 * inv, o1 * inv, o2 * inv, o3 * inv);
    }
}

hipError_t launch_prefill_merge(const PrefillMergeRec *recs, uint32_t n_recs, const float *partials, float *out,
                                const uint32_t *bad, hipStream_t s) {
    if (n_recs == 0)
        return hipSuccess;
    hipLaunchKernelGGL(prefill_merge_kernel, dim3(n_recs, kPrefillCols / 16), dim3(256), 0, s, recs, partials, out, bad);
    return hipGetLastError();
}

// The pool's V rows of one chunk of tokens (all kv heads of one request), as fp16, into the workspace: the
// right-hand side of the one-part product.  Pure copy-and-convert, bound by memory; 16 bytes per lane and pass.
struct V16Args {
    const unsigned char *pool_base;
    uint32_t log2_page;
    const int32_t *page_table;
    const V16Rec *recs;
    unsigned char *v16;
    const uint32_t *bad;
};

__global__ void __launch_bounds__(256) v16_kernel(V16Args a) {
    if (a.bad != nullptr && uni(*reinterpret_cast<const volatile uint32_t *>(a.bad)) != 0)
        return;
    __shared__ V16Rec s_rec;
    if (threadIdx.x == 0)
        s_rec = a.recs[blockIdx.x];
    __syncthreads();
    const uint64_t table_off = uni(s_rec.table_off), T = uni(s_rec.token_bytes);
    const uint32_t t0 = uni(s_rec.t0), t1 = uni(s_rec.t1), ctx_len = uni(s_rec.ctx_len);
    const uint32_t d = uni(s_rec.d), n_kv = uni(s_rec.n_kv);
    unsigned char *dst = a.v16 + uni(s_rec.v16_off);
    const uint32_t lg = a.log2_page;
    const uint64_t page_mask = (1ull << lg) - 1;
    const uint32_t lp = d == 128 ? 4 : 3; // a head's V row has 2^lp 16-byte pieces
    const uint32_t pieces = 1u << lp;
    const uint32_t upt = n_kv * pieces;   // pieces per token
    // the 256 lanes cover whole tokens: several tokens per pass where a token has fewer than 256 pieces
    const uint32_t tid = threadIdx.x;
    uint32_t tstep = 1, tl = 0, r0 = tid, rstep = 256;
    if (upt < 256) {
        tstep = 256 / upt;
        tl = tid / upt;
        r0 = tid % upt;
        rstep = upt;
        if (tl >= tstep)
            return;
    }
    for (uint32_t tok = t0 + tl; tok < t1; tok += tstep) {
        for (uint32_t r = r0; r < upt; r += rstep) {
            const uint32_t h = r >> lp, pc = r & (pieces - 1);
            const uint64_t off = (uint64_t)tok * T + (uint64_t)h * (4 * d) + 2 * d + pc * 16;
            const int32_t pg = as_global(a.page_table)[table_off + (off >> lg)];
            // read once by this pass (the attention kernel takes V from the copy): streaming load; the copy itself
            // is stored plainly, it is read again soon
            const uint4 w = ld_kv(reinterpret_cast<const uint4 *>(a.pool_base + (((uint64_t)(uint32_t)pg << lg) + (off & page_mask))));
            float f[8];
            unpack8(w, f);
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const float x0 = __builtin_amdgcn_fmed3f(f[e], -65504.f, 65504.f);
                const float x1 = __builtin_amdgcn_fmed3f(f[e + 1], -65504.f, 65504.f);
                o[e / 2] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{x0, x1}, f16x2_t));
            }
            *as_global(reinterpret_cast<u32x4 *>(dst + ((uint64_t)h * ctx_len + tok) * (2 * d) + pc * 16)) = (u32x4){o[0], o[1], o[2], o[3]};
        }
    }
}

hipError_t launch_v16(const unsigned char *pool_base, uint32_t log2_page, const int32_t *page_table, const V16Rec *recs,
                      uint32_t n_recs, unsigned char *v16, const uint32_t *bad, hipStream_t s) {
    if (n_recs == 0)
        return hipSuccess;
    V16Args a{pool_base, log2_page, page_table, recs, v16, bad};
    hipLaunchKernelGGL(v16_kernel, dim3(n_recs), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ev0/ev1 (may be null) receive the kernel's own start/stop timestamps.
hipError_t launch_prefill(const PrefillArgs &a, uint32_t n_recs, uint32_t head_dim, uint32_t parts, hipStream_t s,
                          hipEvent_t ev0, hipEvent_t ev1) {
    if (n_recs == 0)
        return hipSuccess;
    static_assert(kPrefillCols == kPrefillWaves * kPrefillBlocks * 16, "NW waves x NB blocks of 16 columns");
    const dim3 grid(n_recs), block(64 * kPrefillWaves);
    if (head_dim == 128 && parts == 1)
        hipExtLaunchKernelGGL((prefill_kernel<kPrefillBlocks, kPrefillWaves, 128, 1>), grid, block, 0, s, ev0, ev1, 0, a);
    else if (head_dim == 128)
        hipExtLaunchKernelGGL((prefill_kernel<kPrefillBlocks, kPrefillWaves, 128, 2>), grid, block, 0, s, ev0, ev1, 0, a);
    else if (parts == 1)
        hipExtLaunchKernelGGL((prefill_kernel<kPrefillBlocks, kPrefillWaves, 64, 1>), grid, block, 0, s, ev0, ev1, 0, a);
    else
        hipExtLaunchKernelGGL((prefill_kernel<kPrefillBlocks, kPrefillWaves, 64, 2>), grid, block, 0, s, ev0, ev1, 0, a);
    return hipGetLastError();
}

} // namespace ukv
