// bf16 MFMA GEMM for gfx950:  C[M, Nn] = A[M, K] * W[Nn, K]^T, fp32 accumulate, fused epilogue.
//
// Both operands are K-contiguous, so each lane's MFMA fragment (8 consecutive k of one
// row) is a single 16-byte LDS read.  A workgroup computes a BM x BN tile with WR x WC
// waves, every wave owning (BM/WR) x (BN/WC) outputs as 16x16 v_mfma_f32_16x16x32_bf16 products
// (a loop of nothing but these sustains 2.1 PFLOP/s on MI355X, the 32x32x16 form 1.85).
// K is consumed 64 at a time through a two-stage LDS ring filled by direct global->LDS
// loads (global_load_lds_dwordx4: no staging registers, no ds_write): the loads of slice
// k+1 are in flight while slice k is multiplied, one barrier per slice.  The A fragments
// of the next 32-deep step are read into the registers of the current ones as soon as
// their MFMAs are issued, the W fragments are double-buffered; LDS reads sit in the
// shadow of the MFMAs.
//
// LDS rows are 128 bytes (64 bf16).  A direct load writes lane j's 16 bytes at
// base + 16*j, so one wave instruction fills 8 rows.  LDS has 64 four-byte banks and a
// 16-byte read is served 16 lanes at a time, so the 16 consecutive rows a fragment read
// touches must land in 16 different 16-byte bank groups: slot p of row r holds chunk
// p ^ ((r >> 1) & 7) (row parity picks the half of the banks, the XOR the group).  The
// swizzle is applied on the global side: lane j of row group g fetches chunk
// (j%8) ^ (4*(g%2) + j/16) of row 8g + j/8.
//
// Epilogue: a 16x16 accumulator gives lane l column l%16 and rows 4*(l/16) + i,
// which would make every store a 2-byte scatter.  Each wave instead passes its tiles, 32 rows
// x 64 columns at a time, through a private LDS patch (row stride 68 floats: conflict-free
// both ways) and reads them back row-contiguous, 4 consecutive columns per lane and 16
// lanes per row.  Bias, GELU, the gated residual update and the rotary rotation then work
// on 16-byte pieces: one 8-byte bf16 store (or 16-byte fp32 store) per 4 outputs, whole
// 128-byte lines per row, the residual / rotary-table operands fetched as 16- / 8-byte loads
// one 32-row strip ahead.
#include "common.h"

namespace ps {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

#define PS_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define PS_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// Consecutive workgroup ids go to different XCDs (8 of them, each with its own L2).
// Give each XCD a contiguous range of tiles so co-resident workgroups share operand panels.
__device__ __forceinline__ int xcd_remap(int id, int total) {
    int per = total / 8, rem = total % 8;
    int x = id % 8, j = id / 8;
    return x * per + (x < rem ? x : rem) + j;
}

// Tile id -> first row and column of the tile.  Tiles walk down the 8 tile rows of a band, column after column, so
// the workgroups resident on one XCD (a contiguous range of ids, about one band) cover a compact block of the
// output and reuse each other's panels in L2.  Each band starts its walk a few columns further on than the one
// before: the XCDs then do not all ask for the same W panel at the same moment (fc1 at 17776 tokens: 8-15 us
// faster inside the network, the other shapes unchanged; larger steps slowed the K-split tail of fc2 down).
__device__ __forceinline__ void tile_origin(int tile, int tiles_m, int tiles_n, int bm, int bn, int& m0, int& n0) {
    constexpr int GM = 8;
    const int per_band = GM * tiles_n;
    const int band = tile / per_band, in_band = tile % per_band;
    const int rows_here = min(GM, tiles_m - band * GM);
    m0 = (band * GM + in_band % rows_here) * bm;
    n0 = ((in_band / rows_here + band * max(1, tiles_n / 8)) % tiles_n) * bn;
}

// tanh-form GELU written as x * sigmoid(2u), u = sqrt(2/pi)(x + 0.044715 x^3): two
// transcendentals and four FMAs; used where the result is rounded to bf16.
__device__ __forceinline__ float gelu_fast(float x) {
    const float c0 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;
    const float c1 = c0 * 0.044715f;
    float t = x * (c0 + c1 * x * x);
    return x * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
}

typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;

constexpr int EPI_LDS_STRIDE = 68;                       // floats per row of a wave's 32 x 64 patch (68 * 4 rows = 16 banks mod 64)
constexpr int EPI_LDS_FLOATS = 32 * EPI_LDS_STRIDE;

// Epilogue of 64 columns of one wave (accumulator tiles J0, J0+1 of each of its TM tile rows): TM strips of
// 32 rows x 64 columns.  wrow0 / wcol0: first row and column of these outputs; patch: the wave's private LDS
// area (EPI_LDS_FLOATS floats).
// Offsets are 32-bit element indices from the uniform base pointers (the launcher
// guarantees M*Nn < 2^31); Nn % 4 == 0, so a lane's 4 columns are inside or outside together.
// The residual values (fp32, 4 consecutive columns) behind output (strip i, row group k) of a wave: rows and
// columns past the edge are clamped (their results are not stored).
__device__ __forceinline__ f32x4_t resid_fetch(const Epilogue& ep, int M, int Nn, int wrow0, int wcol0, int lane, int i, int k) {
    const int rr = lane >> 4, col = wcol0 + (lane & 15) * 4;
    int m = wrow0 + i * 32 + 4 * k + rr;
    m = m < M ? m : M - 1;
    return *reinterpret_cast<const f32x4_t*>(ep.resid + (unsigned)(m * Nn + (col < Nn ? col : 0)));
}

// PRE: `pre` holds the residual values of all TM strips, fetched ahead by the caller, if use_pre (gated residual kind).
template <int TM, int TN, int J0, int KIND, bool CHECK, bool PRE = false, int PN = 1>
__device__ __forceinline__ void wave_epilogue(f32x4_t (&acc)[TM][TN][4], const Epilogue& ep, bf16_t* __restrict__ C,
                                              int M, int Nn, int wrow0, int wcol0, int lane, float* patch,
                                              const f32x4_t (*pre)[8] = nullptr, bool use_pre = false) {
    const int fcol = lane & 15, fgrp = lane >> 4;        // accumulator side: column within 16, row offset 4*fgrp
    const int rr = lane >> 4, cc = (lane & 15) * 4;      // row-contiguous side: row within 4, first column
    const int col = wcol0 + cc;
    const bool col_ok = !CHECK || col < Nn;
    const int colc = col_ok ? col : 0;
    const f32x4_t bias = *reinterpret_cast<const f32x4_t*>(ep.bias + colc);
    const int tokens = ep.geom.tokens, text = ep.geom.text_tokens;
    // batch index of the wave's rows: one division per wave when they share it (the usual case)
    const int row_last = min(wrow0 + TM * 32, M) - 1;
    const int b_first = min(wrow0, M - 1) / tokens;      // (a wave of an edge tile may lie entirely past M)
    const bool one_batch = row_last / tokens == b_first;
    auto token_of = [&](int m, int& b) {
        b = one_batch ? b_first : m / tokens;
        return m - b * tokens;
    };

    // per-kind lane constants
    f32x4_t gate_v = {0.f, 0.f, 0.f, 0.f}, gate_t = gate_v;
    bool rot = false;
    RopeAxis ra0{0, 0, 0}, ra1{0, 0, 0};                 // the lane's two (even, odd) pairs: usually, not always, one axis
    float inv_wp = 0.f, inv_hp = 0.f;
    float qs = 1.0f;
    if constexpr (KIND == EPI_GATE_RESIDUAL) {
        const float* g = ep.mod_layer + b_first * ep.mod_batch_stride + colc;
        gate_v = *reinterpret_cast<const f32x4_t*>(g + ep.gate_chunk * ep.D);
        gate_t = *reinterpret_cast<const f32x4_t*>(g + (ep.gate_chunk + 6) * ep.D);
    }
    if constexpr (KIND == EPI_QKV_ROPE) {
        rot = col < 2 * ep.D;                            // q and k columns rotate, v columns do not
        const int pr = (colc % ep.head_dim) >> 1;        // first of the lane's two pairs
        ra0 = rope_axis_of(pr, ep.head_dim, ep.rope_F, ep.rope_Hp);
        ra1 = rope_axis_of(pr + 1, ep.head_dim, ep.rope_F, ep.rope_Hp);
        inv_wp = 1.0f / (float)ep.rope_Wp;
        inv_hp = 1.0f / (float)ep.rope_Hp;
        qs = col < ep.D ? ep.q_scale : 1.0f;
    }

    // operands the strip needs from memory besides the accumulators (one 16-byte value per
    // 4 outputs): the residual, or (cos, sin, cos, sin) of the two pairs
    auto fetch = [&](int i, int k) -> f32x4_t {
        int m = wrow0 + i * 32 + 4 * k + rr;
        if (CHECK) m = m < M ? m : M - 1;
        if constexpr (KIND == EPI_GATE_RESIDUAL) {
            return *reinterpret_cast<const f32x4_t*>(ep.resid + (unsigned)(m * Nn + colc));
        } else if constexpr (KIND == EPI_QKV_ROPE) {
            int b;
            const int n = token_of(m, b);
            f32x4_t r = {1.f, 0.f, 1.f, 0.f};
            if (rot && n >= text) {
                // video token -> (frame, patch row, patch column); the quotients come from a float multiply and one
                // correction step (exact below 2^22 tokens per sample), then two 8-byte reads of the per-axis table
                // (measured no faster: a copy of the table in LDS and the rows' packed positions computed once per
                // tile, so that this lambda needs neither global loads nor the quotients)
                const int nv = n - text;
                int q1 = (int)((float)nv * inv_wp);
                q1 += (q1 + 1) * ep.rope_Wp <= nv ? 1 : 0;
                q1 -= q1 * ep.rope_Wp > nv ? 1 : 0;
                int q2 = (int)((float)q1 * inv_hp);
                q2 += (q2 + 1) * ep.rope_Hp <= q1 ? 1 : 0;
                q2 -= q2 * ep.rope_Hp > q1 ? 1 : 0;
                const int pj = nv - q1 * ep.rope_Wp, pi = q1 - q2 * ep.rope_Hp;
                const int pos0 = ra0.axis == 0 ? q2 : ra0.axis == 1 ? pi : pj;
                const int pos1 = ra1.axis == 0 ? q2 : ra1.axis == 1 ? pi : pj;
                const f32x2_t a = *reinterpret_cast<const f32x2_t*>(ep.rope_cs + ra0.base + pos0 * ra0.stride);
                const f32x2_t c = *reinterpret_cast<const f32x2_t*>(ep.rope_cs + ra1.base + pos1 * ra1.stride);
                r = f32x4_t{a[0], a[1], c[0], c[1]};
            }
            return r;
        } else {
            return f32x4_t{0.f, 0.f, 0.f, 0.f};
        }
    };
    constexpr bool FETCHES = KIND == EPI_GATE_RESIDUAL || KIND == EPI_QKV_ROPE;

    f32x4_t pf[8];                                       // refilled for the next strip as soon as a value is used
    if constexpr (FETCHES) {
        if (!(PRE && use_pre)) {
#pragma unroll
            for (int k = 0; k < 8; ++k) pf[k] = fetch(0, k);
        }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        // accumulators -> patch (a store instruction covers 4 rows x 16 columns; the row stride puts rows 4
        // apart 16 banks apart: 64 banks)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    patch[(16 * (q >> 1) + 4 * fgrp + e) * EPI_LDS_STRIDE + j * 32 + 16 * (q & 1) + fcol] = acc[i][J0 + j][q][e];
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // LDS is in order per wave; this pins the compiler too
        f32x4_t v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            v[k] = *reinterpret_cast<const f32x4_t*>(patch + (4 * k + rr) * EPI_LDS_STRIDE + cc);
        asm volatile("" ::: "memory");
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int m = wrow0 + i * 32 + 4 * k + rr;
            f32x4_t x = v[k] + bias;
            f32x4_t t = {0.f, 0.f, 0.f, 0.f};
            if constexpr (FETCHES) {
                if (PRE && use_pre) {
                    t = pre[i][k];
                } else {
                    t = pf[k];
                    if (i + 1 < TM) pf[k] = fetch(i + 1, k);
                }
            }
            if constexpr (KIND == EPI_BIAS_GELU) {
#pragma unroll
                for (int c = 0; c < 4; ++c) x[c] = gelu_fast(x[c]);
            }
            if constexpr (KIND == EPI_QKV_ROPE) {
                // t = (cos0, sin0, cos1, sin1); identity for text tokens and v columns
                x = f32x4_t{x[0] * t[0] - x[1] * t[1], x[1] * t[0] + x[0] * t[1],
                            x[2] * t[2] - x[3] * t[3], x[3] * t[2] + x[2] * t[3]} * qs;
            }
            if (CHECK && (m >= M || !col_ok)) continue;
            if constexpr (KIND == EPI_UNPATCHIFY) {
                // token m -> (batch, frame, patch row, patch column); column o -> (channel, dy, dx)
                int b;
                const int n = token_of(m, b);
                if (n < text) continue;
                const PatchGeom& g = ep.pg;
                const int Hp = g.H / g.patch, Wp = g.W / g.patch;
                const int nv = n - text;
                const int pj = nv % Wp, pi = (nv / Wp) % Hp, f = nv / (Wp * Hp);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int o = col + c;
                    const int dx = o % g.patch, dy = (o / g.patch) % g.patch, ch = o / (g.patch * g.patch);
                    ep.resid[((((long)b * g.C + ch) * g.F + f) * g.H + (pi * g.patch + dy)) * g.W + (pj * g.patch + dx)] =
                        x[c];
                }
                continue;
            }
            const unsigned off = (unsigned)(m * Nn + col);
            if constexpr (KIND == EPI_GATE_RESIDUAL) {
                // X[m, col] += gate[batch(m), stream(m), col] * (acc + bias)
                int b;
                const int n = token_of(m, b);
                f32x4_t gate = n < text ? gate_t : gate_v;
                if (!one_batch) {
                    const float* g = ep.mod_layer + b * ep.mod_batch_stride + col;
                    gate = *reinterpret_cast<const f32x4_t*>(g + (ep.gate_chunk + (n < text ? 6 : 0)) * ep.D);
                }
                *reinterpret_cast<f32x4_t*>(ep.resid + off) = t + gate * x;
            } else {
                *reinterpret_cast<bf16x4_t*>(reinterpret_cast<unsigned short*>(C) + off) =
                    __builtin_convertvector(x, bf16x4_t);
            }
        }
    }
}

// global->LDS load of 16 bytes per lane, issued from inline asm: lane j's bytes land at
// lds_addr + 16*j (lds_addr wave-uniform, passed through M0).  The compiler does not see the
// LDS write, so it never orders LDS reads of other stages behind loads still in flight; the
// explicit vmcnt waits and barriers in the kernel make a stage visible before it is read.
__device__ __forceinline__ void lds_dma16(const void* gptr, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr)
                 : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// One BM x BN output tile (rows m0.., columns n0..), k-tiles k0..k1-1 of 64, by the WR x WC waves of a workgroup,
// each owning (BM/WR) x (BN/WC) outputs.  piece >= 0: a K-split piece, accumulators go to ep.split_ws.
// BK: K depth of an LDS stage; NST: ring depth; lds: NST * (BM + BN) * 2 * BK bytes, 1024-aligned.
template <int BM, int BN, int WR, int WC, int BK, int NST, int KIND>
__device__ __forceinline__ void gemm_tile(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, bf16_t* __restrict__ C,
                                          int M, int Nn, int K, int m0, int n0, int k0, int k1, int piece,
                                          const Epilogue& ep, unsigned char* lds) {
    static_assert(BK == 64 || BK == 32, "stage depth");
    constexpr int NW = WR * WC;
    constexpr int WM = BM / WR, WN = BN / WC;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int ROWB = BK * 2;                         // bytes per LDS row
    constexpr int RPI = 1024 / ROWB;                     // rows filled by one wave instruction (8 or 16)
    constexpr int CPR = ROWB / 16;                       // 16-byte chunks per row (8 or 4)
    constexpr int GROUPS = (BM + BN) / RPI;
    constexpr int GPW = GROUPS / NW;                     // load instructions per wave per stage
    constexpr int STAGE = (BM + BN) * ROWB;
    static_assert(TN == 2 || TN == 4, "the epilogue handles strips of 64 columns");
    static_assert(GROUPS % NW == 0, "rows must split evenly over waves");
    static_assert(BM % RPI == 0, "a load group must not straddle the A/W boundary");
    static_assert((NST - 1) * GPW <= 63, "vmcnt range");
    static_assert(NW * EPI_LDS_FLOATS * 4 <= NST * STAGE, "epilogue patches reuse the stage memory");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform values stay in scalar registers
    const int wm = wave / WC, wn = wave % WC;

    // direct loads: lane j of load group g lands at group base + 16j = row RPI*g + j/CPR, slot j%CPR; the slot
    // holds chunk (j%CPR) ^ swizzle(row) of the row (applied on the global side):
    //   128-byte rows: slot p of row r holds chunk p ^ ((r>>1)&7);  64-byte rows: chunk p ^ ((r>>2)&3)
    const int lr = lane / CPR;
    const bf16_t* gp[GPW];
#pragma unroll
    for (int i = 0; i < GPW; ++i) {
        const int g = wave + NW * i;
        const int row = g * RPI + lr;                    // row within [A rows | W rows]
        const int lc = BK == 64 ? ((lane & 7) ^ ((row >> 1) & 7)) : ((lane & 3) ^ ((row >> 2) & 3));
        if (row < BM) {
            int r = m0 + row;
            r = r < M ? r : M - 1;
            gp[i] = A + (long)r * K + lc * 8;
        } else {
            int r = n0 + row - BM;
            r = r < Nn ? r : Nn - 1;
            gp[i] = W + (long)r * K + lc * 8;
        }
    }
    const unsigned lds_base = (unsigned)(size_t)PS_LDS_PTR(lds);
    auto issue_one = [&](int kt, int i) {                // kt counts from k0; ring slot kt % NST; load group i of the wave
        const int kc = k0 + kt < k1 ? k0 + kt : k1 - 1;  // (the prologue of a one-stage piece may ask past the end)
        const unsigned st = lds_base + (kt % NST) * STAGE;
        const int g = wave + NW * i;
        lds_dma16(gp[i] + (long)kc * BK, __builtin_amdgcn_readfirstlane(st + g * 1024));
    };
    auto issue = [&](int kt) {
#pragma unroll
        for (int i = 0; i < GPW; ++i) issue_one(kt, i);
    };
    // (Measured and dropped: a cache prefetch two or four stages ahead of the direct loads -- one 4-byte-per-lane
    // direct load per thread and stage into an LDS area nobody reads, lane r touching the line of row r.  It doubles
    // the cache-line requests through the vector memory path: 8 % slower on the wide shapes, 70 % on K = 7680,
    // with operands cold or warm.)

    // Accumulators: every 32 x 32 block of the wave's outputs is four 16 x 16 products (q = 2 * row half + column
    // half) of v_mfma_f32_16x16x32_bf16, which sustains a higher rate than the 32x32x16 form on this chip
    // (2.1 against 1.85 PFLOP/s in a loop of nothing else).  Lane l of a 16 x 16 result holds column l % 16, rows
    // 4 * (l / 16) .. + 3; of an operand fragment row (or column) l % 16, k = 8 * (l / 16) .. + 7 of a 32-deep step.
    f32x4_t acc[TM][TN][4];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[i][j][q] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    constexpr int FA = 2 * TM, FB = 2 * TN;              // 16-row fragments of A and of W per k-step
    static_assert(BK == 64, "two 32-deep k-steps per stage");
    static_assert(FA >= FB, "the W fragments of the next step are read in the first FB fragment rounds");
    const int l16 = lane & 15, kgrp = lane >> 4;
    int aoff[FA], boff[FB];
#pragma unroll
    for (int x = 0; x < FA; ++x) aoff[x] = (wm * WM + x * 16 + l16) * ROWB;
#pragma unroll
    for (int y = 0; y < FB; ++y) boff[y] = (BM + wn * WN + y * 16 + l16) * ROWB;
    const int sw = (l16 >> 1) & 7;                       // the row offsets above are multiples of 16
    auto slot_of = [&](int ks) { return ((ks * 4 + kgrp) ^ sw) << 4; };

    // A fragments live in one register set: fragment x is read again, for the next k-step, right after the FB
    // MFMAs that consume it (a full k-step before its next use).  W fragments are used by every round of a
    // step, so they are double-buffered.  The one barrier per stage sits in front of the stage's last step,
    // whose operands are already in registers.
    bf16x8_t fa[FA], fb[2][FB];
#pragma unroll
    for (int p = 0; p < NST - 1; ++p) issue(p);
    wait_vmcnt<(NST - 2) * GPW>();                       // own share of stage 0
    __syncthreads();
    issue(NST - 1);
    // Gated residual update on the narrow tile: the residual values of the wave's outputs are requested ahead of
    // the epilogue and sit in registers through the last stages (this tile has registers to spare).  Fetched in the
    // epilogue one strip ahead, their latency was exposed strip by strip: 32 us of the out-projection's 178, 45 us
    // of fc2's 545 at 17776 tokens (measured by leaving the loads out).  Loads return in order, so a wait for a
    // stage's direct loads also waits for every older load: strip 0 is requested right after the last stage's
    // direct loads (third-last iteration), strip 1 after the second-last hand-over, which waits with the 8 loads
    // of strip 0 still allowed in flight; no wait follows until the epilogue.  (Recovers 8 and 15 us.  One request
    // per stage over 16 stages, each allowed to stay out for one hand-over, was 20 us SLOWER: under load a request
    // needs more than a stage to return and then every one of those hand-overs stalls.)
    constexpr bool PRE = KIND == EPI_GATE_RESIDUAL && TN == 2 && TM == 2 && NW == 4;
    f32x4_t pre[PRE ? TM : 1][8];
    const int nkt = k1 - k0;
    const bool have_pre = PRE && piece < 0 && nkt >= 3;
    {
        const int slot = slot_of(0);
#pragma unroll
        for (int x = 0; x < FA; ++x) fa[x] = *reinterpret_cast<const bf16x8_t*>(lds + aoff[x] + slot);
#pragma unroll
        for (int y = 0; y < FB; ++y) fb[0][y] = *reinterpret_cast<const bf16x8_t*>(lds + boff[y] + slot);
    }
    for (int kt = 0; kt < nkt; ++kt) {
        const unsigned char* st = lds + (kt % NST) * STAGE;
        const unsigned char* nx = lds + ((kt + 1) % NST) * STAGE;
        // no stage follows the last one: no hand-over there, and no loads for stages past the end (the fragment
        // reads of the last step then fetch stale, unused data from the other slot)
        const bool more = kt + 1 < nkt, fill = kt + NST < nkt;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const unsigned char* src = st;               // where the next step's fragments come from
            // Direct loads into the slot the barrier frees: one workgroup per CU (8 waves) spreads them over the
            // fragment rounds of the stage's last step (in one block after the barrier they held this wave's MFMAs
            // back for ~30 instructions: QKV / fc1 shapes 6 % faster spread out); with two co-resident workgroups
            // of 4 waves the block form measured 2-3 % faster, the other workgroup covers it.
            constexpr bool SPREAD = NW >= 8;
            if (ks == 1) {
                if (more) {
                    if (PRE && have_pre && kt == nkt - 2) wait_vmcnt<(NST - 2) * GPW + 8>();   // strip 0's loads may stay out
                    else wait_vmcnt<(NST - 2) * GPW>();  // own share of stage kt+1 has landed
                    __syncthreads();                     // ... everyone's; and nobody reads stage kt any more
                }
                if constexpr (!SPREAD) { if (fill) issue(kt + NST); }   // into the slot stage kt occupied
                if constexpr (PRE) {
                    if (have_pre && kt >= nkt - 3 && kt <= nkt - 2) {
                        const bool first = kt == nkt - 3;
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            const f32x4_t v = resid_fetch(ep, M, Nn, m0 + wm * WM, n0 + wn * WN, lane, first ? 0 : 1, k);
                            if (first) pre[0][k] = v; else pre[1][k] = v;
                        }
                    }
                }
                src = nx;
                __builtin_amdgcn_sched_barrier(0);       // hand-over code stays ahead of the MFMAs
            }
            const int slot = slot_of(ks ^ 1);
            if constexpr (!SPREAD) {
#pragma unroll
                for (int x = 0; x < FA; ++x) {
                    if (x < FB) fb[ks ^ 1][x] = *reinterpret_cast<const bf16x8_t*>(src + boff[x] + slot);
#pragma unroll
                    for (int y = 0; y < FB; ++y)
                        acc[x >> 1][y >> 1][(x & 1) * 2 + (y & 1)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            fa[x], fb[ks][y], acc[x >> 1][y >> 1][(x & 1) * 2 + (y & 1)], 0, 0, 0);
                    fa[x] = *reinterpret_cast<const bf16x8_t*>(src + aoff[x] + slot);
                }
#pragma unroll
                for (int x = 0; x < FA; ++x) {           // FB MFMAs, then the LDS reads of the round
                    __builtin_amdgcn_sched_group_barrier(0x008, FB, 0);
                    if (x < FB) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                continue;
            }
            // One fragment round = the FB MFMAs of A fragment x, the LDS reads that refill it (and, in the first
            // rounds, one W fragment of the next step), and in the stage's last step a share of the direct loads.
            constexpr int DPR = (GPW + FA - 1) / FA;     // direct loads per round
#pragma unroll
            for (int x = 0; x < FA; ++x) {
#pragma unroll
                for (int y = 0; y < FB; ++y)
                    acc[x >> 1][y >> 1][(x & 1) * 2 + (y & 1)] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        fa[x], fb[ks][y], acc[x >> 1][y >> 1][(x & 1) * 2 + (y & 1)], 0, 0, 0);
                if (x < FB) fb[ks ^ 1][x] = *reinterpret_cast<const bf16x8_t*>(src + boff[x] + slot);
                fa[x] = *reinterpret_cast<const bf16x8_t*>(src + aoff[x] + slot);
                if (ks == 1 && fill) {
#pragma unroll
                    for (int d = 0; d < DPR; ++d)
                        if (x * DPR + d < GPW) issue_one(kt + NST, x * DPR + d);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    wait_vmcnt<0>();                                     // the look-ahead loads past the end have landed
    __syncthreads();                                     // ... in every wave: the stage memory is free

    if (piece >= 0) {
        // [piece][wave][i][j][lane][16 accumulator registers]
        float* pp = ep.split_ws + (((long)piece * NW + wave) * (TM * TN) * 64 + lane) * 16;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<f32x4_t*>(pp + (i * TN + j) * 64 * 16 + q * 4) = acc[i][j][q];
        return;
    }
    float* patch = reinterpret_cast<float*>(lds) + wave * EPI_LDS_FLOATS;
    const bool interior = (m0 + BM <= M) && (n0 + BN <= Nn);
    if constexpr (PRE) {
        if (interior) wave_epilogue<TM, TN, 0, KIND, false, true>(acc, ep, C, M, Nn, m0 + wm * WM, n0 + wn * WN, lane, patch, pre, have_pre);
        else wave_epilogue<TM, TN, 0, KIND, true, true>(acc, ep, C, M, Nn, m0 + wm * WM, n0 + wn * WN, lane, patch, pre, have_pre);
    } else if (interior) {
        wave_epilogue<TM, TN, 0, KIND, false>(acc, ep, C, M, Nn, m0 + wm * WM, n0 + wn * WN, lane, patch);
        if constexpr (TN == 4)
            wave_epilogue<TM, TN, 2, KIND, false>(acc, ep, C, M, Nn, m0 + wm * WM, n0 + wn * WN + 64, lane, patch);
    } else {
        wave_epilogue<TM, TN, 0, KIND, true>(acc, ep, C, M, Nn, m0 + wm * WM, n0 + wn * WN, lane, patch);
        if constexpr (TN == 4)
            wave_epilogue<TM, TN, 2, KIND, true>(acc, ep, C, M, Nn, m0 + wm * WM, n0 + wn * WN + 64, lane, patch);
    }
}

// Every sample of a batch (rows [b * tokens, (b+1) * tokens) of the operands) is tiled on its own: a tile never
// holds rows of two samples, and which of its tiles are summed in K pieces depends on the sample's shape alone,
// so a sample's result does not depend on the batch it is computed in (Section 3.3: the batched step must
// reproduce the per-step process).  A workgroup shifts the operand, output, residual and modulation
// pointers to its sample and from then on works on a [tokens, Nn] problem.
//
// The first batch * full_tiles workgroups compute one BM x BN output tile each.  The tiles beyond them -- the last,
// partial round of the chip's workgroup slots, per sample -- can be shared out so that the round is shorter: with
// nsplit > 1, nsplit workgroups per tile along K, fp32 partial sums to ep.split_ws (in accumulator layout) for
// gemm_tail_kernel (the narrow tile where K is long).  (Dropped: two workgroups per tail tile of the wide tile,
// one per half of its rows.  With operands resident in the cache from the previous launch it was 2 % faster;
// with weights and activations that change from call to call, as in the network, 1-4 % slower -- each half
// loads the whole W panel again.)
struct GemmGrid { int tokens, batch, tiles_m, tiles_n, full_tiles, tail_tiles, nsplit; };

template <int KIND>
__device__ __forceinline__ void shift_to_sample(Epilogue& ep, int sample, int tokens, int Nn) {
    if constexpr (KIND == EPI_GATE_RESIDUAL) {
        ep.resid += (long)sample * tokens * Nn;
        ep.mod_layer += (long)sample * ep.mod_batch_stride;
    } else if constexpr (KIND == EPI_UNPATCHIFY) {
        ep.resid += (long)sample * ep.pg.C * ep.pg.F * ep.pg.H * ep.pg.W;
    }
}

template <int BM, int BN, int WR, int WC, int BK, int NST, int KIND>
__global__ void __launch_bounds__(WR * WC * 64, (WR * WC == 4 && BM * BN <= 192 * 128) ? 2 : 1)
gemm_mfma_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, bf16_t* __restrict__ C,
                 int Nn, int K, GemmGrid g, Epilogue ep) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[NST * (BM + BN) * BK * 2];
    const int nk = K / BK;
    const int all_full = g.batch * g.full_tiles;
    int sample, tile, piece = -1, k0 = 0, k1 = nk;
    if ((int)blockIdx.x < all_full) {
        const int id = xcd_remap(blockIdx.x, all_full);
        sample = id / g.full_tiles;
        tile = id - sample * g.full_tiles;
    } else {
        piece = blockIdx.x - all_full;                   // index of the partial sums in ep.split_ws
        const int per_sample = g.tail_tiles * g.nsplit;
        sample = piece / per_sample;
        const int lp = piece - sample * per_sample;
        tile = g.full_tiles + lp / g.nsplit;
        const int pi = lp % g.nsplit;
        k0 = nk * pi / g.nsplit;
        k1 = nk * (pi + 1) / g.nsplit;
    }
    sample = __builtin_amdgcn_readfirstlane(sample);
    A += (long)sample * g.tokens * K;
    if (C) C += (long)sample * g.tokens * Nn;
    shift_to_sample<KIND>(ep, sample, g.tokens, Nn);
    int m0, n0;
    tile_origin(tile, g.tiles_m, g.tiles_n, BM, BN, m0, n0);
    gemm_tile<BM, BN, WR, WC, BK, NST, KIND>(A, W, C, g.tokens, Nn, K, m0, n0, k0, k1, piece, ep, lds);
}

// Sums the K-split pieces of the tail tiles (fixed order: deterministic) and applies the epilogue; one single-wave
// workgroup per 32-row strip of each wave of gemm_mfma_kernel's layout (the few tail tiles then spread over 8 to 16
// times as many compute units as they had workgroups: the kernel is a chain of dependent loads).
template <int BM, int BN, int WR, int WC, int KIND>
__global__ void __launch_bounds__(64)
gemm_tail_kernel(bf16_t* __restrict__ C, int Nn, GemmGrid g, Epilogue ep) {
    constexpr int NW = WR * WC;
    constexpr int WM = BM / WR, WN = BN / WC;
    constexpr int TM = WM / 32, TN = WN / 32;
    __shared__ __attribute__((aligned(16))) float patch[EPI_LDS_FLOATS];
    const int lane = threadIdx.x;
    const int strip = blockIdx.x % TM, wave = (blockIdx.x / TM) % NW, tail = blockIdx.x / (TM * NW);   // tail: over all samples
    const int wm = wave / WC, wn = wave % WC;
    const int sample = tail / g.tail_tiles;
    const int tile = g.full_tiles + tail % g.tail_tiles;
    if (C) C += (long)sample * g.tokens * Nn;
    shift_to_sample<KIND>(ep, sample, g.tokens, Nn);
    const int M = g.tokens, nsplit = g.nsplit;
    int m0, n0;
    tile_origin(tile, g.tiles_m, g.tiles_n, BM, BN, m0, n0);
    f32x4_t acc[1][TN][4];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[0][j][q] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    for (int pi = 0; pi < nsplit; ++pi) {
        const float* pp = ep.split_ws + ((((long)tail * nsplit + pi) * NW + wave) * (TM * TN) * 64 + lane) * 16;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                acc[0][j][q] += *reinterpret_cast<const f32x4_t*>(pp + (strip * TN + j) * 64 * 16 + q * 4);
    }
    const int wrow0 = m0 + wm * WM + strip * 32;
    wave_epilogue<1, TN, 0, KIND, true>(acc, ep, C, M, Nn, wrow0, n0 + wn * WN, lane, patch);
    if constexpr (TN == 4)
        wave_epilogue<1, TN, 2, KIND, true>(acc, ep, C, M, Nn, wrow0, n0 + wn * WN + 64, lane, patch);
}

// `tokens` rows per sample; offsets inside a sample are 32-bit element indices
bool gemm_mfma_supported(int tokens, int Nn, int K) {
    return K % 64 == 0 && Nn % 4 == 0 && tokens >= 1 && Nn >= 64 && K >= 64 && (long)tokens * Nn < (1L << 31);
}

// How a sample's [tokens, Nn] output is spread over the chip: which tile variant, how many tiles run whole and
// how the rest is split.  A function of the sample's shape only (never of the batch): see gemm_mfma_kernel.
struct GemmPlan { int variant, bm, bn, per_cu, tiles_m, tiles_n, full, tail, nsplit; size_t ws_bytes_per_sample; };
static int gemm_compute_units() {
    // per device, asked once (a constant of the device, not a setting)
    static int cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int cus = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
        cached[dev] = cus;
    }
    return cached[dev];
}

struct TileVariant { int bm, bn, per_cu; float cost; };
// cost: measured time per output of a full round of workgroup slots, relative to the 256x256 tile, inside the
// 30-layer network at 17776 and 33976 tokens.  The loop is bound by LDS traffic (fragment reads plus the direct
// loads' writes, 128 bytes per clock and CU): a wave tile of 128x64 reads 12 fragments per 32 MFMAs, 96x64 10 per
// 24, 64x64 8 per 16; two co-resident workgroups win some of it back by hiding each other's epilogue.
static const TileVariant kVariants[5] = {
    {0, 0, 0, 0.f},
    {256, 256, 1, 1.00f},     // 1: 8 waves of 128x64
    {128, 128, 2, 1.17f},     // 2: 4 waves of 64x64, two workgroups per CU
    {192, 256, 1, 1.10f},     // 3: 8 waves of 96x64
    {192, 128, 2, 1.10f},     // 4: 4 waves of 96x64, two workgroups per CU
};

// the K split of the last partial round: pieces per tail tile (1: none)
static int tail_split(int tiles, int slots, int K, bool allow_split) {
    const int tail = tiles % slots, nk = K / 64;
    if (!allow_split || K < 4096 || tail == 0 || tiles <= slots) return 1;
    int ns = slots / tail;
    if (ns > 8) ns = 8;
    if (ns > nk / 2) ns = nk / 2;
    return ns >= 2 ? ns : 1;
}

static GemmPlan gemm_plan(int batch, int tokens, int Nn, int K, bool allow_split, int forced_variant) {
    GemmPlan p{};
    const int cus = gemm_compute_units();
    int v = forced_variant;
    if (v < 1 || v > 4) {
        // the variant with the least estimated time: rounds of workgroup slots (a K-split tail counts as 1/pieces of
        // a round plus a fifth of a round for its partial sums and second launch) x tile area x the tile's cost
        // per output.  Outputs with fewer tiles than slots take the smallest tile.
        // Which tiles are summed in K pieces depends on the variant, and must not depend on the batch: where a split
        // is possible (long K) the choice looks at one sample; elsewhere the variant never changes a value and the
        // choice may count the tiles of the whole batch.
        const bool may_split = allow_split && K >= 4096;
        const int nb = may_split ? 1 : batch;
        float best = 0.f;
        v = 2;
        for (int c = 1; c <= 4; ++c) {
            const TileVariant& t = kVariants[c];
            const int tiles = nb * ((tokens + t.bm - 1) / t.bm) * ((Nn + t.bn - 1) / t.bn);
            const int slots = cus * t.per_cu;
            if (tiles < slots) continue;
            const int ns = tail_split(tiles, slots, K, may_split);
            float rounds = (float)(tiles / slots);
            if (tiles % slots) rounds += ns > 1 ? 1.0f / ns + 0.2f : 1.0f;
            const float est = rounds * slots * t.bm * t.bn * t.cost;
            if (best == 0.f || est < best) { best = est; v = c; }
        }
    }
    const TileVariant& t = kVariants[v];
    p.variant = v; p.bm = t.bm; p.bn = t.bn; p.per_cu = t.per_cu;
    p.tiles_m = (tokens + p.bm - 1) / p.bm;
    p.tiles_n = (Nn + p.bn - 1) / p.bn;
    const int tiles = p.tiles_m * p.tiles_n;
    p.full = tiles; p.tail = 0; p.nsplit = 1; p.ws_bytes_per_sample = 0;
    // the last partial round: split along K if the partial sums (two passes over tile-size fp32 per piece) and
    // the second launch cost less than the round they save -- measured at 17776 tokens: true with a long K
    // (fc2 on 128x128 tiles: 0.62 -> 0.57 ms), not for K = 1920 (0.188 -> 0.196 ms)
    const int slots = cus * p.per_cu;
    const int ns = tail_split(tiles, slots, K, allow_split);
    if (ns > 1) {
        const int tail = tiles % slots;
        p.full = tiles - tail; p.tail = tail; p.nsplit = ns;
        p.ws_bytes_per_sample = (size_t)tail * ns * p.bm * p.bn * sizeof(float);
    }
    return p;
}

// kernel path: low byte = mode (4: never split a tail along K), bits 8-11 = forced tile variant (0: automatic)
static int forced_variant_of(int path) { return (path >> 8) & 0xf; }

size_t gemm_split_workspace_bytes(int dtype, int batch, int tokens, int Nn, int K, int path) {
    if (dtype != PS_BF16 || !gemm_mfma_supported(tokens, Nn, K) || (path & 0xff) == 4) return 0;
    return gemm_plan(batch, tokens, Nn, K, true, forced_variant_of(path)).ws_bytes_per_sample * (size_t)batch;
}

template <int BM, int BN, int WR, int WC, int BK, int NST, int KIND>
static hipError_t launch_kind(const bf16_t* A, const bf16_t* W, bf16_t* C, int batch, int tokens, int Nn, int K,
                              const GemmPlan& p, const Epilogue& ep, hipStream_t st) {
    dim3 block(WR * WC * 64);
    const GemmGrid g{tokens, batch, p.tiles_m, p.tiles_n, p.full, p.tail, p.nsplit};
    const int grid = batch * (p.full + p.tail * p.nsplit);
    gemm_mfma_kernel<BM, BN, WR, WC, BK, NST, KIND><<<grid, block, 0, st>>>(A, W, C, Nn, K, g, ep);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.tail == 0) return e;
    gemm_tail_kernel<BM, BN, WR, WC, KIND><<<batch * p.tail * (WR * WC) * (BM / WR / 32), 64, 0, st>>>(C, Nn, g, ep);
    return hipGetLastError();
}

template <int BM, int BN, int WR, int WC, int BK, int NST>
static hipError_t launch_tile(const bf16_t* A, const bf16_t* W, bf16_t* C, int batch, int tokens, int Nn, int K,
                              const GemmPlan& p, const Epilogue& ep, hipStream_t st) {
    switch (ep.kind) {
        case EPI_BIAS: return launch_kind<BM, BN, WR, WC, BK, NST, EPI_BIAS>(A, W, C, batch, tokens, Nn, K, p, ep, st);
        case EPI_BIAS_GELU: return launch_kind<BM, BN, WR, WC, BK, NST, EPI_BIAS_GELU>(A, W, C, batch, tokens, Nn, K, p, ep, st);
        case EPI_GATE_RESIDUAL: return launch_kind<BM, BN, WR, WC, BK, NST, EPI_GATE_RESIDUAL>(A, W, C, batch, tokens, Nn, K, p, ep, st);
        case EPI_QKV_ROPE: return launch_kind<BM, BN, WR, WC, BK, NST, EPI_QKV_ROPE>(A, W, C, batch, tokens, Nn, K, p, ep, st);
        case EPI_UNPATCHIFY: return launch_kind<BM, BN, WR, WC, BK, NST, EPI_UNPATCHIFY>(A, W, C, batch, tokens, Nn, K, p, ep, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gemm_mfma(const bf16_t* A, const bf16_t* W, bf16_t* C, int batch, int tokens, int Nn, int K,
                            const Epilogue& ep, int path, hipStream_t st) {
    const bool tails = (path & 0xff) != 4;
    const int fv = forced_variant_of(path);
    GemmPlan p = gemm_plan(batch, tokens, Nn, K, ep.split_ws != nullptr && tails, fv);
    if (p.ws_bytes_per_sample * (size_t)batch > ep.split_ws_bytes) p = gemm_plan(batch, tokens, Nn, K, false, fv);
    switch (p.variant) {
        case 1: return launch_tile<256, 256, 2, 4, 64, 2>(A, W, C, batch, tokens, Nn, K, p, ep, st);   // 8 waves, 128x64 each
        case 2: return launch_tile<128, 128, 2, 2, 64, 2>(A, W, C, batch, tokens, Nn, K, p, ep, st);   // 4 waves, 64x64 each, 2 per CU
        case 3: return launch_tile<192, 256, 2, 4, 64, 2>(A, W, C, batch, tokens, Nn, K, p, ep, st);   // 8 waves, 96x64 each
        case 4: return launch_tile<192, 128, 2, 2, 64, 2>(A, W, C, batch, tokens, Nn, K, p, ep, st);   // 4 waves, 96x64 each, 2 per CU
        // Measured and dropped: 4 waves of 128x128 outputs on the 256x256 tile (fewer LDS reads per MFMA; with the
        // 32x32x16 MFMA one wave per SIMD issued one only every ~48 cycles: 5-15 % slower; with 16x16x32 the 256
        // accumulator registers per lane make the compiler shuttle values between the two register files, 3-4
        // copies per MFMA: 30 % slower; with the MFMAs written as inline asm on accumulator-file operands the
        // copies go, and the variant is the fastest at 8192 x 8192 weights, 1.28 PFLOP/s, but 5-10 % slower than
        // the 8-wave tile at this model's shapes: one wave per SIMD has nobody to cover its barrier waits);
        // 32-deep stages in rings of 3 or 4
        // (5-25 % slower: twice the barriers).  With the loads of the loop taken out (timing probe) both tiles
        // reach 1.3-1.4 PFLOP/s, with every tile loading the same L2-resident panels only 4-10 % more than now:
        // the global->LDS path itself, not the memory behind L2, is what the loop waits for (a stand-alone stream
        // of such loads delivers 47 bytes per clock and CU; global_load + ds_write_b128 delivers 70, but staging
        // the stages through registers made the real loop 5-12 % slower on both tiles).
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ps
