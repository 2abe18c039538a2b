// Marching SpMM over the stored CSR arrays with the entry stream staged through LDS.
//
// Why a second marching kernel.  In spmm_march_kernel (apply_march_kernel.h) eight lanes share a
// row and load its entries as 32-byte pieces; its counters at batch 16 show the vector ALUs busy
// about four cycles in five while waves are resident, and per 8 rows it issues some 320 vector
// instructions of which 112 are the multiply-adds: the lanes pay the address arithmetic for 56
// slots of a 49-entry row, the eight partial sums cost a 42-instruction reduce-scatter per row
// group, and the accumulators are cleared for every row.  Fewer lanes per row would cure all
// three, but then a wave's 4-byte loads would touch 64 / G different memory lines per instruction
// and come back to each line in later instructions, which the 32 KB vector L1 does not survive
// (a one-lane-per-row variant that loaded 8 entries per row at a time ran at 165 us with the
// arithmetic removed).  So here the loads and the arithmetic use different lane layouts:
//
//  * loads: the entries of a wave's 64 / G consecutive rows are one contiguous span of col_idx and
//    of vals.  The wave loads that span with 16 bytes per lane, every instruction one contiguous
//    kilobyte, every memory line touched exactly once (buffer loads: a wave-uniform descriptor that
//    ends with the span, so a lane past its end fetches nothing and reads zero), one whole pass ahead of the
//    arithmetic, and writes the registers into an LDS image of the span at the end of the pass;
//  * arithmetic: G lanes share a row, lane l takes entries l, l+G, ... of it from the LDS image
//    (4-byte LDS reads at compile-time offsets), computes the LDS address of the stored column in
//    the ring of input lines exactly as spmm_march_kernel does (an entry whose column is not on a
//    resident line -- possible only if the arrays were edited -- is taken from global memory),
//    reads the pixel's NV float4 chunks and does 4*NV multiply-adds.  With G = 2 a 49-entry row
//    costs 50 slots and one DPP add per accumulator.
//
// Work mapping.  A workgroup of 8 waves owns a strip of 32 output columns and a segment of output
// lines and walks down it WL lines per step; a wave owns 64 / G neighbouring rows of one line
// (G = 2: a whole line of the strip, WL = 8; G = 4: half a line, WL = 4; G = 8: a quarter, WL = 2;
// G = 16 compiles too but measured slower than G = 8 where both fit).
// The input lines the step can touch sit in a ring of NL LDS lines (slot = line mod NL), one
// plane per float4 chunk of batch columns; the lines the next step adds travel global ->
// registers during the step and registers -> LDS between the two barriers that end it.  Every
// load of a step -- entries, row bounds, input lines -- is issued at its start and first used
// at its end, so nothing waits for memory while there is arithmetic left.
//
// Several input channels (MC).  The channels share row_ptr and col_idx and have a vals array and
// an x plane each; y is their sum.  A step is then one block of WL result lines for ONE channel,
// the channels of a block in turn: the accumulators stay in registers from the first channel of
// the block to the last, after which the lanes combine and store as usual -- y is written once,
// never read, and the sum has a fixed order.  The image keeps the block's columns while the
// channels pass (only the values are loaded again), and the ring is refilled with the whole
// window of the next channel's plane instead of the lines a block adds.
#pragma once
#include <type_traits>

#include "apply_march_kernel.h"

namespace convspmv {

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}), written out
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, I + 1>(f);
    }
}

constexpr int kStageTw = 32;                 // output columns per strip
constexpr int kStageWaves = 8;

// bytes of LDS a wave needs for its image of NLD * 256 entries (col_idx and vals)
constexpr int stage_wave_bytes(int nld) { return nld * 256 * 8; }
// LDS pixels per ring plane: what the images leave of a CU's 160 KiB, shared by the planes
// (NV float4 planes, or one plane of floats), at most 4612, rounded down to 4 mod 16 so that
// the planes start 16 banks apart
constexpr int stage_plane(int nv, int nld) {
    const int left = 160 * 1024 - kStageWaves * stage_wave_bytes(nld);
    const int px = left / (nv ? nv * 16 : 4);
    const int capped = px > 4612 ? 4612 : px;
    return (capped - 4) / 16 * 16 + 4;
}

// G: lanes per row (2, 4, 8).  NIT: entries per lane, ceil(longest row / G).  NV: float4 column
// chunks per lane (0: one scalar column).  NL: ring lines (power of two, at least the lines WL
// output lines can touch).  XLD: registers per thread that carry the next step's input lines.
// NLD: 16-byte loads per lane, array and pass; NLD * 256 >= (64 / G) * longest row + 3.
// CS: LDS pixels per plane (> NL * iw_pitch).  MC: walk g.channels input channels per block of lines.
template <int G, int NIT, int NV, int NL, int XLD, int NLD, int CS, bool MC = false>
__global__ __launch_bounds__(kWave *kStageWaves) void spmm_stage_march_kernel(const int *__restrict__ row_ptr,
                                                                            const int *__restrict__ col_idx,
                                                                            const float *__restrict__ vals,
                                                                            const float *__restrict__ x,
                                                                            float *__restrict__ y, MarchGeom g) {
    constexpr bool SCALAR = NV == 0;
    constexpr int NP = SCALAR ? 1 : NV;           // LDS planes
    constexpr int NVAL = SCALAR ? 1 : 4 * NV;     // batch columns per lane
    constexpr int SH = SCALAR ? 2 : 4;            // log2 of the LDS bytes per pixel and plane
    constexpr int PIXB = 1 << SH;
    using elem_t = typename std::conditional<SCALAR, float, vec4>::type;
    constexpr int NTHREADS = kWave * kStageWaves;
    constexpr int TW = kStageTw;
    constexpr int RW = kWave / G;                 // rows per wave
    constexpr int WC = TW / RW;                   // waves per output line
    constexpr int WL = kStageWaves / WC;          // output lines per step
    constexpr int CAP = NLD * 256;                // entries the wave's image holds
    constexpr int SCAT = ilog2(G) < ilog2(NVAL) ? ilog2(G) : ilog2(NVAL);
    constexpr int CNT = NVAL >> SCAT;             // finished columns per storing lane
    constexpr int DUP = ilog2(G) - SCAT;          // low lane bits that end up with copies
    typedef int ivec4 __attribute__((ext_vector_type(4)));
    static_assert(G == 2 || G == 4 || G == 8 || G == 16, "lanes per row");
    static_assert((NL & (NL - 1)) == 0, "ring size");
    static_assert(NIT * G + 7 <= CAP && RW * ((NIT - 1) * G + 1) + 3 <= CAP, "image too small for the rows");
    extern __shared__ float4 smem[];
    elem_t *xs = reinterpret_cast<elem_t *>(smem);   // [NP planes][CS pixels]

    // ---- which strip segment and block of batch columns (as in spmm_march_kernel)
    const int turn = blockIdx.x / kXcds;
    const int local = turn / g.col_blocks, col_block = turn - local * g.col_blocks;
    const int job = (blockIdx.x % kXcds) * g.blocks_per_xcd + local;
    if (local >= g.blocks_per_xcd || job >= g.strips * g.segs) return;      // uniform over the block
    const int sg = job / g.strips, tx = job - sg * g.strips;
    const int y0 = tx * TW, xa = sg * g.seg, xb = min(xa + g.seg, g.m_out);
    const int twc = min(TW, g.n_out - y0);
    const int c0 = col_block * NVAL;
    const int tid = threadIdx.x, lane = tid % kWave;
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int gl = lane % G, gr = lane / G;
    const int wline = wave / WC;                  // this wave's line within a step
    const int wcol = (wave % WC) * RW;            // first strip column of this wave's rows
    const int nch = MC ? g.channels : 1;

    char *lds_tail = reinterpret_cast<char *>(smem) + (size_t)NP * CS * PIXB;
    int *img_c = reinterpret_cast<int *>(lds_tail + wave * stage_wave_bytes(NLD));   // image of the wave's span of col_idx
    float *img_v = reinterpret_cast<float *>(img_c + CAP);                           // ... and of vals

    // ---- operand columns of the strip, clipped to the image
    auto first_window = [&](int t) {
        const int num = t + g.p - g.k + 1;
        return num > 0 ? (num + g.s - 1) / g.s : 0;
    };
    const int j_lo = g.tr ? first_window(y0) : g.s * y0 - g.p;
    const int j0 = min(max(j_lo, 0), g.n - 1);
    const int iwc = max(min(j_lo + g.iw, g.n) - j0, 0);
    const float inv_iwc = 1.0f / (float)max(iwc, 1);
    const int zslot = NL * g.iw_pitch;            // a pixel of zeros in every plane

    // first / one-past-last operand line that result lines [xo, xo + cnt) can touch, clipped
    auto line_lo = [&](int xo) { return min(max(g.tr ? first_window(xo) : g.s * xo - g.p, 0), g.m); };
    auto line_hi = [&](int xo, int cnt) {
        const int last = xo + cnt - 1;
        return min(max(g.tr ? (last + g.p) / g.s + 1 : g.s * last - g.p + g.k, 0), g.m);
    };

    // ---- the loads of one pass of this wave (result line xo): the span of its rows' entries,
    // 16 bytes per lane and instruction, and the bounds of this lane's row
    struct PassLoads {
        ivec4 c[NLD];
        ivec4 v[NLD];             // bit patterns of the values
        int beg, end;             // row_ptr of this lane's row
    };
    // first row of the wave on line xo (clamped into the segment, so that every address is valid)
    auto wave_row = [&](int xo) { return (long long)min(xo, xb - 1) * g.n_out + y0 + min(wcol, twc - 1); };
    // first entry of the wave's span on line xo: a wave-uniform address, so a scalar load
    // ... and one past its last entry (the end of the last row the wave has on that line)
    struct Span { int beg, end; };
    auto span_of = [&](int xo) {
        const long long r0 = wave_row(xo);
        const int nrows = min(max(twc - wcol, 1), RW);
        return Span{__builtin_amdgcn_readfirstlane(row_ptr[r0]), __builtin_amdgcn_readfirstlane(row_ptr[r0 + nrows])};
    };
    // The loads of a pass are issued piece by piece between the rounds of the arithmetic of the
    // pass before (see compute): a wave that issues them in one go sits in the issue of its
    // 2 * NLD + 2 load instructions until the memory pipeline has taken all of them, which is most
    // of the time their bytes need, and computes nothing meanwhile (measured: the time of the
    // loads and the time of the arithmetic added up).
    struct SetInfo {                      // what land() must know of a pass, kept beside its register set
        int sb4;                          // first entry of the column image (span begin rounded down to 16 bytes)
        int dv;                           // image index of an entry in the value image minus that in the column image
        int ch;                           // channel of the pass
    };
    struct IssueState {
        __amdgpu_buffer_rsrc_t rc, rv;    // wave-uniform descriptors of the span, from its first entry (rounded down to 16 bytes) to its end
        long long row;                    // this lane's row (clamped into the segment)
    };
    constexpr int NPIECE = 2 * NLD + 2;
    // Cache policy of the entry loads.  Every line is used once, so non-temporal loads (which the
    // L2 drops first) keep x resident; but the memory system moves more when the traffic is a mix
    // of both kinds: with all entry loads non-temporal the headline product takes 98.8 us, with
    // none 108 us, with two of the seven kilobytes per array and pass loaded normally 91 us; at
    // batch 1, where x is 1 % of the bytes, three of seven are best (73.8 -> 66.1 us; four: 70.8,
    // all: 79 us).  About 35-40 % of all bytes on the normal path, that is: the first NCACHED
    // pieces of each array.
    constexpr int kStreamAux = 2;
    // (several channels: every step reloads its whole window of x with normal loads, and no mix of
    // the entry loads measured better than all of them non-temporal.  Eight lanes per row: the
    // shapes that take them have long rows and, at 4096^2, k 11, s 4, batch 4, x is a fifth of the
    // bytes: none 205 us, one of four 216, two 217, three 220.)
    // Four lanes per row (1024^2, k 9, batch 16): none 162 us, one of seven 156, two 168, three 171.
    constexpr int NCACHED = (MC || G >= 8) ? 0 : G == 4 ? 1 : (NLD * (NV == 4 ? 29 : 43) + 50) / 100;
    auto issue_begin = [&](int xo, int ch, Span sp, IssueState &st, SetInfo &si) {
        const int sb4 = sp.beg & ~3;                                 // 16-byte aligned
        // the descriptors end where the span ends: lanes past it fetch nothing and read zeros
        // (the image holds a multiple of 256 entries, up to a seventh more than a span)
        // (a line past the segment's end -- the loads run two steps ahead of the arithmetic -- has an
        // empty span: nothing is fetched for it)
        const int end = xo < xb ? min(sp.end, g.nnz) : sb4;
        const int bytes = max(end - sb4, 0) * 4;
        // the values of channel ch start ch * nnz entries further on; their image is aligned on its own
        const long long vabs = (MC ? (long long)ch * g.nnz : 0) + sp.beg;
        const long long vb4 = vabs & ~3LL;
        const int vbytes = MC ? (xo < xb ? max((int)(vabs - sp.beg + end - vb4), 0) * 4 : 0) : bytes;
        si.sb4 = sb4;
        si.dv = MC ? (int)(vabs - vb4) - (sp.beg - sb4) : 0;
        si.ch = ch;
        constexpr int kRsrcFlags = 0x00020000;                       // raw buffer of 32-bit elements, gfx9 encoding
        // (the columns are those of the block: loaded with its first channel only)
        st.rc = __builtin_amdgcn_make_buffer_rsrc(const_cast<int *>(col_idx + sb4), 0, (MC && ch != 0) ? 0 : bytes, kRsrcFlags);
        st.rv = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(vals + vb4), 0, vbytes, kRsrcFlags);
        st.row = wave_row(xo) + min(gr, max(twc - 1 - wcol, 0));
    };
    auto issue_piece = [&](auto p_tag, const IssueState &st, PassLoads &pl) {
        constexpr int P = decltype(p_tag)::value;
        if constexpr (P < 2 * NLD) {
            constexpr int i = P / 2;
            constexpr int AUX = i < NCACHED ? 0 : kStreamAux;
            if constexpr (P % 2 == 0) pl.c[i] = __builtin_amdgcn_raw_buffer_load_b128(st.rc, lane * 16, i * 1024, AUX);
            else pl.v[i] = __builtin_amdgcn_raw_buffer_load_b128(st.rv, lane * 16, i * 1024, AUX);
        } else if constexpr (P == 2 * NLD) {
            pl.beg = row_ptr[st.row];
        } else {
            pl.end = row_ptr[st.row + 1];
        }
    };
    auto issue = [&](int xo, int ch, Span sp, PassLoads &pl, SetInfo &si) {   // all pieces at once (before the march)
        IssueState st;
        issue_begin(xo, ch, sp, st, si);
        static_for<NPIECE>([&](auto p_tag) { issue_piece(p_tag, st, pl); });
    };
    // registers -> the wave's LDS image; the row of this lane: position of its first entry in the
    // image (plus the lane's slot) and its length
    int pos = 0, len = 0, vshift = 0;
    auto land = [&](int xo, const PassLoads &pl, const SetInfo &si) {
        ivec4 *dc = reinterpret_cast<ivec4 *>(img_c) + lane;
        ivec4 *dv = reinterpret_cast<ivec4 *>(img_v) + lane;
        if (!MC || si.ch == 0) {
#pragma unroll
            for (int i = 0; i < NLD; ++i) dc[i * kWave] = pl.c[i];
        }
#pragma unroll
        for (int i = 0; i < NLD; ++i) dv[i * kWave] = pl.v[i];
        const bool valid = xo < xb && wcol + gr < twc;
        len = valid ? pl.end - pl.beg : 0;
        pos = pl.beg - si.sb4 + gl;
        vshift = si.dv;
        // a row the image does not hold (only arrays edited beyond the documented row length
        // can do that) is cut off at the image's end
        if (pos + min(vshift, 0) < 0 || pos + max(vshift, 0) + (NIT - 1) * G >= CAP) pos = 3, len = 0;
    };

    // ---- window state of this wave's line (wave-uniform), in bytes of LDS as in spmm_march_kernel:
    // dB = PIXB * (col - cbase) = PIXB * (di * n + dj) for a column on line ibase + di at strip
    // pixel dj; ibase is a multiple of NL, so the ring slot of the line is di % NL.  The host
    // guarantees m*n <= 2^27 and 2*NL*n*16 <= 2^25, which keeps dB exact in fp32 and the quotient
    // by n exact after one fused multiply-add and a truncation.
    const int nB = g.n * PIXB, pitchB = g.iw_pitch * PIXB, zslotB = zslot * PIXB;
    const unsigned iwcB = (unsigned)iwc * PIXB;
    const float inv_nB = g.inv_n / (float)PIXB, half_inv_n = 0.5f * g.inv_n;
    int cbaseB = 0, loB = 0, neg_cbaseB = 0;
    unsigned spanB = 0;
    // (-n * PIXB and -cbaseB as values of their own: added in a shift-add and a multiply-add, where
    // the compiler otherwise subtracts first and pays an instruction more per slot)
    int neg_nB = -nB;
    asm volatile("" : "+s"(neg_nB));
    auto set_window = [&](int xo) {
        const int lo = line_lo(xo), hi = line_hi(xo, 1);
        const int ibase = lo & ~(NL - 1);
        cbaseB = (ibase * g.n + j0) * PIXB;
        neg_cbaseB = -cbaseB;
        asm volatile("" : "+s"(neg_cbaseB));
        loB = (lo - ibase) * nB;
        spanB = (unsigned)(hi - lo) * (unsigned)nB;
    };
    auto fma_elem = [](float *a, float wt, const elem_t &e) {
        if constexpr (SCALAR) {
            a[0] = fmaf(wt, e, a[0]);
        } else {
            a[0] = fmaf(wt, e.x, a[0]);
            a[1] = fmaf(wt, e.y, a[1]);
            a[2] = fmaf(wt, e.z, a[2]);
            a[3] = fmaf(wt, e.w, a[3]);
        }
    };

    // ---- one pass: the lane's NIT slots of its row, then the G partial sums combined and stored.
    // Between the rounds the pieces of the loads two steps ahead are issued into `nw`.
    float acc[NVAL];                     // (MC: carried from the first channel of a block of lines to the last)
    const float *xcur = x;               // the plane of the channel being computed
    auto compute = [&](int xo, const IssueState &st, PassLoads &nw, bool first, bool last) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NVAL; ++i) acc[i] = (!MC || first) ? 0.0f : acc[i];
        bool stray = false;              // an in-row entry whose column is not on a resident line
        // A slot is four steps, each fed by the one before: (A) read the stored column and value
        // from the image, (B) turn the column into an LDS address and the value into a weight,
        // (C) read the pixel there, (D) multiply-add.  A workgroup fills the LDS of its CU, so a
        // SIMD has two waves and nobody else to hide an LDS round trip: the steps of a slot are
        // spread over four rounds instead -- round t does A of slot t + 3, B of slot t + 2, C of
        // slot t + 1 and D of slot t, which do not depend on each other.  The rounds are written
        // out (every register has a compile-time name: slot mod 4, pixel set slot mod 2) and
        // kept in one basic block, in this order, by the scheduling barriers.
        const int *pc = img_c + pos;
        const float *pv = img_v + pos + vshift;
        const int rem = len - gl;                    // slot t belongs to the row iff t * G < rem
        int cc[4], addr[4];
        float vv[4], w[4];
        elem_t xq[2][NP];
        auto step_a = [&](int t) {
            cc[t & 3] = pc[t * G];
            vv[t & 3] = pv[t * G];
        };
        auto step_b = [&](int t) {
            const int u = t & 3;
            const bool act = t * G < rem;
            const int dB = (cc[u] << SH) + neg_cbaseB;
            const int di = (int)fmaf((float)dB, inv_nB, half_inv_n);
            const int djB = __mul24(di, neg_nB) + dB;
            const bool in = (unsigned)(dB - loB) < spanB && (unsigned)djB < iwcB;
            stray |= act && !in;
            int a = __mul24(di & (NL - 1), pitchB) + djB;
            // (computed whether or not it is used: a conditional computation would split the block)
            asm volatile("" : "+v"(a));
            addr[u] = (act && in) ? a : zslotB;
            w[u] = (act && in) ? vv[u] : 0.0f;
        };
        auto step_c = [&](int t) {
            const elem_t *src = reinterpret_cast<const elem_t *>(reinterpret_cast<const char *>(xs) + addr[t & 3]);
#pragma unroll
            for (int v = 0; v < NP; ++v) xq[t & 1][v] = src[v * CS];
        };
        auto step_d = [&](int t) {
#pragma unroll
            for (int v = 0; v < NP; ++v) fma_elem(acc + 4 * v, w[t & 3], xq[t & 1][v]);
        };
        step_a(0);
        if constexpr (NIT > 1) step_a(1);
        if constexpr (NIT > 2) step_a(2);
        step_b(0);
        if constexpr (NIT > 1) step_b(1);
        step_c(0);
        static_for<NIT>([&](auto t_tag) {
            constexpr int t = decltype(t_tag)::value;
            if constexpr (t + 3 < NIT) step_a(t + 3);
            if constexpr (t + 2 < NIT) step_b(t + 2);
            if constexpr (t + 1 < NIT) step_c(t + 1);
            __builtin_amdgcn_sched_barrier(0);
            step_d(t);
            // the pieces of the next loads that fall to this round
            static_for<NPIECE>([&](auto p_tag) {
                constexpr int P = decltype(p_tag)::value;
                if constexpr (P * NIT / NPIECE == t) issue_piece(p_tag, st, nw);
            });
            __builtin_amdgcn_sched_barrier(0);
        });
        if (__builtin_expect(__any(stray), 0)) {
            // cold: some stored column is not on a resident line; take those from global memory
            // (the entries are read from the image again: keeping NIT columns and values in
            // registers for this path would cost the hot path its registers)
            asm volatile("" ::: "memory");
#pragma unroll 1
            for (int t = 0; t < NIT; ++t) {
                const int c = img_c[pos + t * G];
                const float v = img_v[pos + vshift + t * G];
                const bool act = t * G + gl < len;
                const int dB = (c << SH) - cbaseB;
                const int di = (int)fmaf((float)dB, inv_nB, half_inv_n);
                const int djB = dB - __mul24(di, nB);
                const bool in = (unsigned)(dB - loB) < spanB && (unsigned)djB < iwcB;
                if (act && !in) {
                    const elem_t *src = reinterpret_cast<const elem_t *>(xcur + (long long)c * g.batch + c0);
#pragma unroll
                    for (int q = 0; q < NP; ++q) fma_elem(acc + 4 * q, v, src[q]);
                }
            }
        }

        if (MC && !last) return;         // (uniform) more channels of this block to come
        // ---- combine the G partial sums of each row; all 64 lanes are active here
        if constexpr (G == 16) {
            combine_step<NVAL, kDppXor15>(acc, (gl & 8) != 0);
            combine_step<imax(NVAL / 2, 1), kDppXor7>(acc, (gl & 4) != 0);
            combine_step<imax(NVAL / 4, 1), kDppXor2>(acc, (gl & 2) != 0);
            combine_step<imax(NVAL / 8, 1), kDppXor1>(acc, (gl & 1) != 0);
        } else if constexpr (G == 8) {
            combine_step<NVAL, kDppXor7>(acc, (gl & 4) != 0);
            combine_step<imax(NVAL / 2, 1), kDppXor2>(acc, (gl & 2) != 0);
            combine_step<imax(NVAL / 4, 1), kDppXor1>(acc, (gl & 1) != 0);
        } else if constexpr (G == 4) {
            combine_step<NVAL, kDppXor2>(acc, (gl & 2) != 0);
            combine_step<imax(NVAL / 2, 1), kDppXor1>(acc, (gl & 1) != 0);
        } else {
            combine_step<NVAL, kDppXor1>(acc, (gl & 1) != 0);
        }
        // lanes whose DUP low bits are clear hold CNT finished columns of their row,
        // starting at column (gl >> DUP) * CNT of this launch's column block
        if constexpr (CNT == 8) {
            // Two 16-byte pieces per lane: stored directly, an instruction would write every
            // other piece of each memory line.  Through the wave's image instead (its entries
            // are used up): afterwards lane l holds piece l of the wave's rows, and each store
            // instruction writes 64 consecutive pieces.
            vec4 *sc = reinterpret_cast<vec4 *>(img_c);
            vec4 q0, q1;
            q0.x = acc[0]; q0.y = acc[1]; q0.z = acc[2]; q0.w = acc[3];
            q1.x = acc[4]; q1.y = acc[5]; q1.z = acc[6]; q1.w = acc[7];
            wave_lds_order();
            sc[lane * 2] = q0;
            sc[lane * 2 + 1] = q1;
            wave_lds_order();
            constexpr int QPR = NVAL / 4;                // pieces per row
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int q = i * kWave + lane;
                const vec4 t = sc[q];
                const int row = wcol + q / QPR, part = q % QPR;
                if (xo < xb && row < twc) {
                    float *dst = y + ((long long)xo * g.n_out + (y0 + row)) * g.batch + c0 + part * 4;
                    float out[4] = {t.x, t.y, t.z, t.w};
                    store_row<4>(dst, out, g.accum != 0);
                }
            }
            wave_lds_order();
        } else {
            const int yy = wcol + gr;
            if (xo < xb && yy < twc && (gl & ((1 << DUP) - 1)) == 0) {
                float *dst = y + ((long long)xo * g.n_out + (y0 + yy)) * g.batch + c0 + (gl >> DUP) * CNT;
                store_row<CNT>(dst, acc, g.accum != 0);
            }
        }
    };

    // ---- operand lines of the next step: global -> registers now, registers -> LDS between the
    // two barriers that end the step.  Always XLD loads per thread (clamped addresses).
    elem_t xr[XLD];
    int xdst[XLD];                       // LDS pixel index, or -1
    auto load_next_lines = [&](int xo_next, const float *xplane) {
        // the lines the block at xo_next adds to the one before (MC: its whole window, of another plane)
        const int lo = MC ? line_lo(xo_next) : line_hi(xo_next - WL, WL), hi = line_hi(xo_next, WL);
        const int items = xo_next < xb ? (hi - lo) * iwc * NP : 0;
#pragma unroll
        for (int r = 0; r < XLD; ++r) {
            const int item = tid + r * NTHREADS;
            const int q = item / NP, v = item % NP;
            const int dl = div_small(q, inv_iwc), dj = min(q - dl * iwc, max(iwc - 1, 0));
            const int i = min(lo + dl, g.m - 1);
            const elem_t *src = reinterpret_cast<const elem_t *>(xplane + ((long long)i * g.n + (j0 + dj)) * g.batch + c0);
            xr[r] = src[v];
            xdst[r] = item < items ? v * CS + (i & (NL - 1)) * g.iw_pitch + dj : -1;
        }
    };
    auto store_next_lines = [&]() {
#pragma unroll
        for (int r = 0; r < XLD; ++r)
            if (xdst[r] >= 0) xs[xdst[r]] = xr[r];
    };

    // ---- the march.  Step q is result lines xa + P*WL .. + WL-1 (this wave's: xa + P*WL + wline) of
    // channel c, with P = q / channels and c = q mod channels (one channel: P = q).
    // While step q is computed from the LDS image, the loads of step q + 1 are in flight and those
    // of step q + 2 are issued (two register sets, so the loop is written two steps per round; an
    // odd count runs one step more, on lines past the segment's end, which holds no row and
    // stores nothing): memory never waits for the arithmetic or for the exchange at the end of a step.
    const int npass = (xb - xa + WL - 1) / WL;             // uniform over the workgroup
    const int nsteps = npass * nch;
    struct At { int blk, ch; };                            // first line of a step's block, its channel
    auto after = [&](At a) {
        if (!MC || a.ch + 1 == nch) return At{a.blk + WL, 0};
        return At{a.blk, a.ch + 1};
    };
    auto plane = [&](int ch) { return MC ? x + (long long)ch * g.x_plane : x; };
    const At at0{xa, 0}, at1 = after(at0), at2 = after(at1);
    PassLoads pl_a, pl_b;
    SetInfo si_a, si_b;
    issue(at0.blk + wline, 0, span_of(at0.blk + wline), pl_a, si_a);
    {   // lines of the first step -> LDS
        const int lo = line_lo(xa), hi = line_hi(xa, WL);
        const int items = (hi - lo) * iwc * NP;
        for (int item = tid; item < items; item += NTHREADS) {
            const int q = item / NP, v = item % NP;
            const int dl = div_small(q, inv_iwc), dj = q - dl * iwc;
            const int i = lo + dl;
            const elem_t *src = reinterpret_cast<const elem_t *>(x + ((long long)i * g.n + (j0 + dj)) * g.batch + c0);
            xs[v * CS + (i & (NL - 1)) * g.iw_pitch + dj] = src[v];
        }
        if (tid < NP) xs[tid * CS + zslot] = elem_t(0.0f);
    }
    land(at0.blk + wline, pl_a, si_a);
    issue(at1.blk + wline, at1.ch, span_of(at1.blk + wline), pl_b, si_b);
    Span sp_next = span_of(at2.blk + wline);               // requested a step ahead of the loads that start there
    At cur = at0, nxt = at1, nxt2 = at2;
    __syncthreads();

    // one step: the loads of step q + 2 go into `nw`, those of step q + 1 land from `old`
    auto step = [&](PassLoads &nw, SetInfo &si_nw, const PassLoads &old, const SetInfo &si_old) __attribute__((always_inline)) {
        const int xo = cur.blk + wline;
        // the ring lines first: they are needed at the end of this step, the entries a step later
        load_next_lines(nxt.blk, plane(nxt.ch));
        IssueState st;
        issue_begin(nxt2.blk + wline, nxt2.ch, sp_next, st, si_nw);
        const At nxt3 = after(nxt2);
        sp_next = span_of(nxt3.blk + wline);
        set_window(xo);
        xcur = plane(cur.ch);
        __builtin_amdgcn_sched_barrier(0);
        compute(xo, st, nw, cur.ch == 0, cur.ch == nch - 1);
        __builtin_amdgcn_sched_barrier(0);
        // the wave's own image first (its LDS instructions execute in order, the reads of this
        // step are done), the ring lines once every wave has left the step
        land(nxt.blk + wline, old, si_old);
        __syncthreads();
        store_next_lines();
        __syncthreads();
        cur = nxt, nxt = nxt2, nxt2 = nxt3;
    };
    for (int q = 0; q < nsteps; q += 2) {
        step(pl_a, si_a, pl_b, si_b);
        if (MC || q + 1 < nsteps) step(pl_b, si_b, pl_a, si_a);
    }
}

}  // namespace convspmv
