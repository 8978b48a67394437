// GQA decode attention over the mixed KV set (bf16, matrix cores): split-KV partials and the
// fixed-order log-sum-exp merge.
//
// The G*T query rows that share one KV head (G = query heads per KV head) are stacked along the
// query dimension: row rho = t*G + hg.  A workgroup owns one (query b, KV head g, row tile,
// key split) and streams its slice of Kmix/Vmix exactly once through LDS (64-key tiles, double
// buffered, next tile prefetched into registers); every wave owns QB blocks of 32 query rows.
// Each workgroup writes a normalised partial output and the base-2 log-sum-exp of its scaled
// logits; the merge kernel combines the splits of a row with weights and a summation order
// that depend only on the split index, so the result does not depend on scheduling.
#include "vxl_internal.h"
#include "vxl_mfma.h"

namespace vxl {

namespace {

template <int D, int QB>
struct DecodeCfg {
    static constexpr int RT = 128 * QB;            // query rows per workgroup
    static constexpr int KROW = LdsRows<D>::K;     // LDS row strides (elements)
    static constexpr int VROW = LdsRows<D>::V;
    static constexpr int K_ELEMS = kKeyTile * KROW;
    static constexpr int V_ELEMS = kKeyTile * VROW;
    static constexpr int LDS_BYTES = 2 * (K_ELEMS + V_ELEMS) * 2;
};

// Row map of the in-place form (IND instances of the kernels below): the mixed KV set is not a
// buffer but a list of rows -- mixed row r of query b is token src_idx[b, r] of the dense K / V
// (KV head g at kv_head elements, rows kv_tok elements apart) or, if negative, row -1 - src_idx of
// the sparse buffers Ksp / Vsp [Hkv, S_total, D].
struct RowMap {
    const int32_t* src_idx;     // [B, l_cap]
    const uint16_t* Ksp;        // may be null when no entry is negative
    const uint16_t* Vsp;
    long long kv_head;          // elements
    long long kv_tok;           // elements
    int s_total;
};

template <int D, int QB, bool IND = false>
__global__ __launch_bounds__(256, (QB == 1 ? 2 : 1)) void decode_split_kernel(
    const uint16_t* __restrict__ Qd, const uint16_t* __restrict__ Kmix, const uint16_t* __restrict__ Vmix,
    const int32_t* __restrict__ mix_len, float* __restrict__ part_o, float* __restrict__ part_lse, int T_q,
    int n_q_heads, int n_kv_heads, int group, int l_cap, int n_rtile, int split_len, float scale, RowMap rm) {
    using C = DecodeCfg<D, QB>;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    uint16_t* Ks = lds;
    uint16_t* Vs = lds + 2 * C::K_ELEMS;

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: scalar control flow
    const int split = blockIdx.x, n_split = gridDim.x;
    const int g = blockIdx.y % n_kv_heads, rt = blockIdx.y / n_kv_heads;
    const int b = blockIdx.z;
    const int n_rows = group * T_q;
    const int len = min(max(mix_len[b], 0), l_cap);
    const int k_lo = split * split_len;
    const int k_hi = min(k_lo + split_len, len);
    const int wrow0 = rt * C::RT + wave * 32 * QB;
    const size_t part_base = (((size_t)b * n_kv_heads + g) * n_split + split) * (size_t)n_rows;

    if (k_lo >= k_hi) {                            // empty split: only its weight (zero) is recorded
        for (int r = rt * C::RT + tid; r < min(n_rows, (rt + 1) * C::RT); r += 256)
            part_lse[part_base + r] = -INFINITY;
        return;
    }

    bf16x8 qreg[QB][D / 16];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int rho = min(wrow0 + qb * 32 + l32, n_rows - 1);
        const int t = rho / group, hg = rho % group;
        const uint4* src = (const uint4*)(Qd + (((size_t)b * T_q + t) * n_q_heads + g * group + hg) * D);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qreg[qb][ks] = __builtin_bit_cast(bf16x8, src[ks * 2 + hi]);
    }
    f32x16 o[QB][D / 32];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < D / 32; ++db) o[qb][db] = zero16();
    }
    const float c2 = scale * kLog2e;
    const bool wave_active = wrow0 < n_rows;       // waves without rows only help with the copies

    // (IND: Kmix / Vmix are the dense K / V of the layer, read through the row map)
    const char* kbase = IND ? (const char*)(Kmix + (size_t)g * rm.kv_head)
                            : (const char*)(Kmix + ((size_t)b * n_kv_heads + g) * (size_t)l_cap * D);
    const char* vbase = IND ? (const char*)(Vmix + (size_t)g * rm.kv_head)
                            : (const char*)(Vmix + ((size_t)b * n_kv_heads + g) * (size_t)l_cap * D);
    const long long ksp_delta = IND ? (const char*)(rm.Ksp + (size_t)g * rm.s_total * D) - kbase : 0;
    const long long vsp_delta = IND ? (const char*)(rm.Vsp + (size_t)g * rm.s_total * D) - vbase : 0;
    const int32_t* src_b = IND ? rm.src_idx + (size_t)b * l_cap : nullptr;
    const int ld_r = tid / (D / 8), ld_part = tid % (D / 8);
    TileRegs<D, C::VROW> tr;
    const int n_t = (k_hi - k_lo + kKeyTile - 1) / kKeyTile;
    // rows past the end of the split are clamped to its last row (scores masked, V finite)
    // IND: the rows of tile t are fetched through the map entries loaded one call earlier, and the
    // entries of tile t + 1 (clamped to the last tile) are requested in the same call
    auto load_map = [&](int key0_) {
        tr.load_map(src_b + key0_, ld_r, min(kKeyTile - 1, k_hi - 1 - key0_));
    };
    auto fetch = [&](int key0_, int key0_after_) {
        const int rlim_ = min(kKeyTile - 1, k_hi - 1 - key0_);
        if constexpr (IND) {
            tr.fetch_mapped(kbase, vbase, ksp_delta, vsp_delta, rm.kv_tok * 2, ld_part);
            load_map(key0_after_);
        } else {
            tr.fetch(kbase + (size_t)key0_ * (D * 2), vbase + (size_t)key0_ * (D * 2), ld_r, ld_part, rlim_);
        }
    };
    if constexpr (IND) load_map(k_lo);
    fetch(k_lo, k_lo + min(1, n_t - 1) * kKeyTile);
    tr.stage(Ks, Vs, ld_r, ld_part);
    __syncthreads();
    for (int ti = 0; ti < n_t; ++ti) {
        const int buf = ti & 1;
        const int key0 = k_lo + ti * kKeyTile;
        {   // next tile (the last iteration re-reads its own): unconditional, fenced, in flight below
            fetch(k_lo + min(ti + 1, n_t - 1) * kKeyTile, k_lo + min(ti + 2, n_t - 1) * kKeyTile);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (wave_active) {
            f32x16 s[QB][2];
            qk_tile<D, QB, C::KROW>(Ks + buf * C::K_ELEMS, qreg, l32, hi, s);
            if (key0 + kKeyTile > k_hi) {
                const int lim = k_hi - key0 - 1;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            s[qb][kb][r] = acc_key(kb, r, hi) <= lim ? s[qb][kb][r] : -INFINITY;
            }
            bf16x8 pb[QB][2][2];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                softmax_tile<D / 32>(s[qb], c2, m_run[qb], l_run[qb], o[qb], pb[qb]);
            pv_tile<D, QB, C::VROW>(Vs + buf * C::V_ELEMS, pb, lane, o);
        }
        tr.stage(Ks + (buf ^ 1) * C::K_ELEMS, Vs + (buf ^ 1) * C::V_ELEMS, ld_r, ld_part);
        __syncthreads();
    }

    if (!wave_active) return;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int rho = wrow0 + qb * 32 + l32;
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
        if (rho >= n_rows) continue;
        const float inv = 1.f / l_tot;
        float* orow = part_o + (part_base + rho) * D;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                float4 v;
                v.x = o[qb][db][rq * 4 + 0] * inv;
                v.y = o[qb][db][rq * 4 + 1] * inv;
                v.z = o[qb][db][rq * 4 + 2] * inv;
                v.w = o[qb][db][rq * 4 + 3] * inv;
                *(float4*)(orow + db * 32 + rq * 8 + hi * 4) = v;
            }
        if (hi == 0) part_lse[part_base + rho] = m_run[qb] * c2 + __builtin_amdgcn_logf(l_tot);
    }
}

// ------------------------------------------------------------------------------------------
// Batched kernel for more than 128 stacked query rows: 256 rows and 8 waves per workgroup (one row
// block of 32 per wave, two waves per SIMD), the split's 64-key tiles streamed into a ring of NS
// LDS stages by direct global->LDS loads, two tiles ahead of the arithmetic -- the structure of
// the streaming pre-filling kernel, without its causal part.  The loads are issued from inline
// assembly and counted by hand (every wave issues the same number per tile and waits with
// vmcnt = loads still allowed in flight), so the kernel must not spill, and the query registers
// are forced complete before the first ring load.  Same partials as decode_split_kernel.
// ------------------------------------------------------------------------------------------
template <int D, int NS>
struct DecodeRingCfg {
    static constexpr int WAVES = 8;
    static constexpr int RT = 32 * WAVES;                     // query rows per workgroup
    static constexpr int TILE = kKeyTile * D;                 // elements of one unpadded K (or V) tile
    static constexpr int STAGE = 2 * TILE;                    // K tile then V tile
    static constexpr int LDS_BYTES = NS * STAGE * 2;
    static constexpr int PPR = D / 8;                         // 16-byte pieces per row
    static constexpr int RPI = 64 / PPR;                      // rows per load instruction (1 KiB)
    static constexpr int NI = kKeyTile / RPI;                 // instructions per tile per matrix
    static constexpr int IPW = NI / WAVES;                    // ... per wave
    static constexpr int GROUP = 2 * IPW;                     // loads per wave per tile (K and V)
};

// IND (in-place form): the rows of a tile are reached through the row map.  A lane needs one map
// entry per load slot and tile; the entries of tiles t+2, t+3 are fetched (by loads issued from
// inline assembly, so that they ride in the hand-kept vmcnt count) when the loads of tiles t, t+1 are
// issued, and are complete behind the same vmcnt(0) that tiles t, t+1 wait for.
template <int D, int NS, bool IND = false>
__global__ __launch_bounds__(512, 2) void decode_ring_kernel(
    const uint16_t* __restrict__ Qd, const uint16_t* __restrict__ Kmix, const uint16_t* __restrict__ Vmix,
    const int32_t* __restrict__ mix_len, float* __restrict__ part_o, float* __restrict__ part_lse, int T_q,
    int n_q_heads, int n_kv_heads, int group, int l_cap, int n_rtile, int split_len, float scale, RowMap rm) {
    using C = DecodeRingCfg<D, NS>;
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int split = blockIdx.x, n_split = gridDim.x;
    const int g = blockIdx.y % n_kv_heads, rt = blockIdx.y / n_kv_heads;
    const int b = blockIdx.z;
    const int n_rows = group * T_q;
    const int len = __builtin_amdgcn_readfirstlane(min(max(mix_len[b], 0), l_cap));
    const int k_lo = split * split_len;
    const int k_hi = min(k_lo + split_len, len);
    const int wrow0 = rt * C::RT + wave * 32;
    const size_t part_base = (((size_t)b * n_kv_heads + g) * n_split + split) * (size_t)n_rows;

    if (k_lo >= k_hi) {                            // empty split: only its weight (zero) is recorded
        for (int r = rt * C::RT + tid; r < min(n_rows, (rt + 1) * C::RT); r += 512)
            part_lse[part_base + r] = -INFINITY;
        return;
    }
    const int n_t = (k_hi - k_lo + kKeyTile - 1) / kKeyTile;
    // (IND: Kmix / Vmix are the dense K / V of the layer)
    const char* kbase = IND ? (const char*)(Kmix + (size_t)g * rm.kv_head)
                            : (const char*)(Kmix + (((size_t)b * n_kv_heads + g) * (size_t)l_cap + k_lo) * D);
    const char* vbase = IND ? (const char*)(Vmix + (size_t)g * rm.kv_head)
                            : (const char*)(Vmix + (((size_t)b * n_kv_heads + g) * (size_t)l_cap + k_lo) * D);
    const long long ksp_delta = IND ? (const char*)(rm.Ksp + (size_t)g * rm.s_total * D) - kbase : 0;
    const long long vsp_delta = IND ? (const char*)(rm.Vsp + (size_t)g * rm.s_total * D) - vbase : 0;
    const long long kv_tok_bytes = IND ? rm.kv_tok * 2 : 0;
    const int32_t* src_s = IND ? rm.src_idx + (size_t)b * l_cap + k_lo : nullptr;      // map entries of this split
    const int r_in = lane / C::PPR, pp = lane % C::PPR;

    // IND: map entries of this lane's load slots for one tile
    struct TileMap { int e[C::IPW]; };
    auto load_map = [&](int t, TileMap& m) __attribute__((always_inline)) {
        const int row0 = t * kKeyTile;
        const int rlim = min(kKeyTile - 1, k_hi - k_lo - 1 - row0);
#pragma unroll
        for (int i = 0; i < C::IPW; ++i)
            m.e[i] = load_i32_hidden(src_s + row0 + min((wave + i * C::WAVES) * C::RPI + r_in, rlim));
    };
    // Tile t -> stage t % NS.  Every wave issues GROUP loads: instruction slots wave, wave + 8, ...
    // Rows past the end of the split are clamped to its last row (scores masked, V finite).
    auto issue = [&](int t, const TileMap& m) __attribute__((always_inline)) {
        const int row0 = t * kKeyTile;
        const int rlim = min(kKeyTile - 1, k_hi - k_lo - 1 - row0);
        const char* kb = kbase + (size_t)row0 * (D * 2);
        const char* vb = vbase + (size_t)row0 * (D * 2);
        const uint32_t st = lds_base + (uint32_t)(t % NS) * (C::STAGE * 2);
#pragma unroll
        for (int i = 0; i < C::IPW; ++i) {
            const int slot = wave + i * C::WAVES;
            const int row = slot * C::RPI + r_in;
            const int kp = pp ^ ((row / (16 / C::PPR)) & (C::PPR - 1));
            constexpr int CPR = D * 2 / 64, RPL = D == 128 ? 1 : 2;
            const int vp = (((pp >> 2) ^ ((row / RPL) & (CPR - 1))) << 2) | (pp & 3);
            if constexpr (IND) {
                const long long ko = mapped_row_offset(m.e[i], kv_tok_bytes, D * 2, ksp_delta);
                const long long vo = mapped_row_offset(m.e[i], kv_tok_bytes, D * 2, vsp_delta);
                dma16_addr(kbase + ko + kp * 16, st + slot * 1024);
                dma16_addr(vbase + vo + vp * 16, st + C::TILE * 2 + slot * 1024);
            } else {
                const uint32_t roff = (uint32_t)min(row, rlim) * (D * 2);
                dma16(kb, roff + kp * 16, st + slot * 1024);
                dma16(vb, roff + vp * 16, st + C::TILE * 2 + slot * 1024);
            }
        }
    };
    // Two groups of TPB stages: one is consumed while the other is refilled, one workgroup barrier
    // per TPB tiles.
    constexpr int TPB = 2;
    static_assert(NS == 2 * TPB, "two groups of TPB stages");
    TileMap ma{}, mb{};                                       // entries of the next two tiles to be issued
    if constexpr (IND) {
        load_map(0, ma);
        load_map(min(1, n_t - 1), mb);
        wait_vmcnt<0>();
#pragma unroll
        for (int i = 0; i < C::IPW; ++i) { settle_i32(ma.e[i]); settle_i32(mb.e[i]); }
    }
    issue(0, ma);
    issue(min(1, n_t - 1), mb);
    if constexpr (IND) {                                      // entries of tiles 2, 3: complete behind the first meeting's wait
        load_map(min(2, n_t - 1), ma);
        load_map(min(3, n_t - 1), mb);
    }

    // Query rows: loaded after the ring has been started (the latencies overlap) and forced
    // complete here; from here on no load the compiler knows of is outstanding.
    bf16x8 qreg[1][D / 16];
    {
        const int rho = min(wrow0 + l32, n_rows - 1);
        const int t = rho / group, hg = rho % group;
        const uint4* src = (const uint4*)(Qd + (((size_t)b * T_q + t) * n_q_heads + g * group + hg) * D);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qreg[0][ks] = __builtin_bit_cast(bf16x8, src[ks * 2 + hi]);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
            typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
            asm volatile("" :: "v"(__builtin_bit_cast(u32x4, qreg[0][ks])));
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    f32x16 o[1][D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) o[0][db] = zero16();
    float m_run = -INFINITY, l_run = 0.f;
    const float c2 = scale * kLog2e;
    const bool wave_active = wrow0 < n_rows;       // waves without rows only help with the loads

    auto process = [&](int ti) {
        if (!wave_active) return;
        const uint16_t* kt = lds + (ti % NS) * C::STAGE;
        const int key0 = k_lo + ti * kKeyTile;
        f32x16 s[1][2];
        qk_tile<D, 1, D>(kt, qreg, l32, hi, s);
        if (key0 + kKeyTile > k_hi) {
            const int lim = k_hi - key0 - 1;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[0][kb][r] = acc_key(kb, r, hi) <= lim ? s[0][kb][r] : -INFINITY;
        }
        bf16x8 pb[1][2][2];
        softmax_tile<D / 32>(s[0], c2, m_run, l_run, o[0], pb[0]);
        pv_tile<D, 1, D>(kt + C::TILE, pb, lane, o);
    };
    for (int t0 = 0; t0 < n_t; t0 += TPB) {
        wait_vmcnt<0>();                                      // this wave's parts of tiles t0, t0+1 have landed
        __builtin_amdgcn_s_barrier();                         // ... and everyone's; the other group is free
        if constexpr (IND) {
#pragma unroll
            for (int i = 0; i < C::IPW; ++i) { settle_i32(ma.e[i]); settle_i32(mb.e[i]); }
        }
        issue(min(t0 + TPB, n_t - 1), ma);
        if constexpr (IND) load_map(min(t0 + 2 * TPB, n_t - 1), ma);
        process(t0);
        issue(min(t0 + TPB + 1, n_t - 1), mb);
        if constexpr (IND) load_map(min(t0 + 2 * TPB + 1, n_t - 1), mb);
        if (t0 + 1 < n_t) process(t0 + 1);
    }
    wait_vmcnt<0>();                                          // drain the refills before the wave ends

    if (!wave_active) return;
    const int rho = wrow0 + l32;
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (rho >= n_rows) return;
    const float inv = 1.f / l_tot;
    float* orow = part_o + (part_base + rho) * D;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
            float4 v;
            v.x = o[0][db][rq * 4 + 0] * inv;
            v.y = o[0][db][rq * 4 + 1] * inv;
            v.z = o[0][db][rq * 4 + 2] * inv;
            v.w = o[0][db][rq * 4 + 3] * inv;
            *(float4*)(orow + db * 32 + rq * 8 + hi * 4) = v;
        }
    if (hi == 0) part_lse[part_base + rho] = m_run * c2 + __builtin_amdgcn_logf(l_tot);
}

// ------------------------------------------------------------------------------------------
// Step-mode kernel for at most 32 stacked query rows (e.g. T = 1..4 at G = 7): the work is pure
// streaming, so every WAVE owns its own 32-key tiles (tile = NW*(split*tpw + i) + wave) and its
// own LDS tile pairs, filled by direct global->LDS loads; there is no workgroup barrier in the
// loop.  The waves' running (reference, sum, O) are merged through LDS in wave order and the
// workgroup writes one normalised partial + base-2 LSE per row.
// Two forms, both filling 128 KiB of LDS: NW = 4 waves with two tile pairs each -- the next tile
// is requested before the current one is worked on, so a wave waits for memory once, not once per
// tile (the default: 3-8 % faster on long streams, 5 % at a single tile per wave, where it spreads
// over twice as many compute units) -- and NW = 8 waves with one tile pair each (cross-check).
constexpr int kStepTile = 32;       // keys per wave tile
constexpr int kMaxStepTpw = 32;     // in-place form: tiles per wave whose row map fits the wave's LDS area

template <int D, int NW, int NBUF, bool IND = false>
__global__ __launch_bounds__(64 * NW, 2) void decode_wave_kernel(
    const uint16_t* __restrict__ Qd, const uint16_t* __restrict__ Kmix, const uint16_t* __restrict__ Vmix,
    const int32_t* __restrict__ mix_len, float* __restrict__ part_o, float* __restrict__ part_lse, int T_q,
    int n_q_heads, int n_kv_heads, int group, int l_cap, int tiles_per_wave, float scale, RowMap rm) {
    static_assert(!IND || NBUF == 2, "the in-place form exists for the double-buffered kernel only");
    constexpr int TK = kStepTile;
    constexpr int TILE_ELEMS = TK * D;                         // one unpadded tile
    extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
    __shared__ float stats[NW][32][2];                         // per wave and row: reference logit, sum
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    uint16_t* Kw = lds + wave * NBUF * 2 * TILE_ELEMS;         // this wave's K tile, then its V tile (NBUF times)
    uint16_t* Vw = Kw + TILE_ELEMS;
    const int split = blockIdx.x, n_split = gridDim.x, g = blockIdx.y, b = blockIdx.z;
    const int n_rows = group * T_q;                            // <= 32
    const int len = min(max(mix_len[b], 0), l_cap);
    const int n_tiles = (len + TK - 1) / TK;
    const size_t part_base = (((size_t)b * n_kv_heads + g) * n_split + split) * (size_t)n_rows;

    const float c2 = scale * kLog2e;
    // (IND: Kmix / Vmix are the dense K / V of the layer, read through the row map)
    const char* kbase = IND ? (const char*)(Kmix + (size_t)g * rm.kv_head)
                            : (const char*)(Kmix + ((size_t)b * n_kv_heads + g) * (size_t)l_cap * D);
    const char* vbase = IND ? (const char*)(Vmix + (size_t)g * rm.kv_head)
                            : (const char*)(Vmix + ((size_t)b * n_kv_heads + g) * (size_t)l_cap * D);
    const int tile0 = split * tiles_per_wave * NW + wave;      // this wave's tiles: tile0, tile0 + NW, ...
    // IND: the source rows of this wave's tiles go to LDS first (ordinary loads, complete before the
    // first hand-counted request), so that the requests depend on LDS reads only.
    __shared__ int32_t row_src[IND ? NW * kMaxStepTpw * TK : 1];
    int32_t* src_w = row_src + (IND ? wave * kMaxStepTpw * TK : 0);
    // byte distances from the dense to the sparse buffers (one base per tensor keeps the addresses in registers)
    const long long ksp_delta = IND ? (const char*)(rm.Ksp + (size_t)g * rm.s_total * D) - kbase : 0;
    const long long vsp_delta = IND ? (const char*)(rm.Vsp + (size_t)g * rm.s_total * D) - vbase : 0;
    const long long kv_tok_bytes = IND ? rm.kv_tok * 2 : 0;
    if constexpr (IND) {
        // (all entries up to the capacity, so that these loads do not wait for the length; entries at
        // and past the length may be anything and are never turned into addresses: request() clamps the
        // row index to the last valid one before it reads the map)
        const int32_t* src_b = rm.src_idx + (size_t)b * l_cap;
        for (int i = 0; i < tiles_per_wave; ++i) {
            const int tile = tile0 + i * NW;
            if (tile * TK >= l_cap) break;
            if (lane < TK) src_w[i * TK + lane] = src_b[min(tile * TK + lane, l_cap - 1)];
        }
        __builtin_amdgcn_s_waitcnt(0x0070);                    // vmcnt(0) lgkmcnt(0): the map is in LDS
        __builtin_amdgcn_wave_barrier();
    }

    // NBUF == 2: direct loads issued from inline assembly and counted by hand (a later request
    // must be allowed to stay in flight while an earlier tile is read).
    constexpr int PPR = D / 8, RPI = 64 / PPR, NL = TK / RPI;  // pieces per row; rows, 1 KiB lines per tile
    const uint32_t lds_w = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)Kw;
    // i_ = position of the tile among this wave's tiles (its row map is src_w + i_ * TK)
    // n_valid = rows that may be read: the mixed length, or (gathered form, first request only) the
    // capacity of the buffers, so that the first request does not wait for the load of the length.
    auto request = [&](int i_, int tile_, int buf, int n_valid) __attribute__((always_inline)) {
        const int key0_ = tile_ * TK;
        const int rlim_ = min(TK - 1, n_valid - 1 - key0_);
        const char* kb = kbase + (size_t)key0_ * (D * 2);
        const char* vb = vbase + (size_t)key0_ * (D * 2);
        const int r_in = lane / PPR, pp = lane % PPR;
        int src_row[NL];                                       // IND: source row of this lane's row in every load
        if constexpr (IND) {
            // rows x * RPI + r_in, clamped to the last valid one: a constant stride except at the clamp
            const uint32_t base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)(src_w + i_ * TK);
            // A full tile whose 32 entries are consecutive rows of one source (a dense chunk: e0, e0 + 1,
            // ...; the sparse buffer: e0, e0 - 1, ...) is fetched like a tile of a gathered buffer, from
            // one scalar base with 32-bit lane offsets: the same number of loads, far fewer instructions.
            if (rlim_ == TK - 1) {
                int ent[1];
                lds_read_i32_hidden<1>(base + (lane & (TK - 1)) * 4, 0, ent);
                const int e0 = __builtin_amdgcn_readfirstlane(ent[0]);
                const int step = e0 >= 0 ? 1 : -1;
                if (kv_tok_bytes < (1ll << 26) &&                // (32 rows x stride must fit the 32-bit lane offset)
                    __builtin_amdgcn_ballot_w64(ent[0] != e0 + step * (lane & (TK - 1))) == 0) {
                    const char* kb1 = kbase + mapped_row_offset(e0, kv_tok_bytes, D * 2, ksp_delta);
                    const char* vb1 = vbase + mapped_row_offset(e0, kv_tok_bytes, D * 2, vsp_delta);
                    const uint32_t row_bytes = e0 >= 0 ? (uint32_t)kv_tok_bytes : (uint32_t)(D * 2);
#pragma unroll
                    for (int x = 0; x < NL; ++x) {
                        const int row = x * RPI + r_in;
                        const int kp = pp ^ ((row / (16 / PPR)) & (PPR - 1));
                        constexpr int CPR = D * 2 / 64, RPL = D == 128 ? 1 : 2;
                        const int vp = (((pp >> 2) ^ ((row / RPL) & (CPR - 1))) << 2) | (pp & 3);
                        const uint32_t kdst = lds_w + (uint32_t)buf * (4 * TILE_ELEMS) + x * 1024;
                        dma16(kb1, (uint32_t)row * row_bytes + kp * 16, kdst);
                        dma16(vb1, (uint32_t)row * row_bytes + vp * 16, kdst + 2 * TILE_ELEMS);
                    }
                    return;
                }
            }
            if (rlim_ == TK - 1) {
                lds_read_i32_hidden<NL>(base + r_in * 4, RPI * 4, src_row);
            } else {
#pragma unroll
                for (int x = 0; x < NL; ++x) {
                    int one[1];
                    lds_read_i32_hidden<1>(base + min(x * RPI + r_in, rlim_) * 4, 0, one);
                    src_row[x] = one[0];
                }
            }
        }
#pragma unroll
        for (int x = 0; x < NL; ++x) {
            const int row = x * RPI + r_in;
            const int kp = pp ^ ((row / (16 / PPR)) & (PPR - 1));
            constexpr int CPR = D * 2 / 64, RPL = D == 128 ? 1 : 2;
            const int vp = (((pp >> 2) ^ ((row / RPL) & (CPR - 1))) << 2) | (pp & 3);
            const uint32_t kdst = lds_w + (uint32_t)buf * (4 * TILE_ELEMS) + x * 1024;
            const uint32_t vdst = kdst + 2 * TILE_ELEMS;
            if constexpr (IND) {
                const long long ko = mapped_row_offset(src_row[x], kv_tok_bytes, D * 2, ksp_delta);
                const long long vo = mapped_row_offset(src_row[x], kv_tok_bytes, D * 2, vsp_delta);
                dma16_addr(kbase + ko + kp * 16, kdst);
                dma16_addr(vbase + vo + vp * 16, vdst);
            } else {
                const uint32_t roff = (uint32_t)min(row, rlim_) * (D * 2);
                dma16(kb, roff + kp * 16, kdst);
                dma16(vb, roff + vp * 16, vdst);
            }
        }
    };
    if constexpr (NBUF == 2) {
        // Gathered form: rows up to the capacity are readable memory whatever the length turns out
        // to be (rows past it are masked when the tile is worked on, and a wave without tiles drains
        // the request before the merge), so tile 0 is requested before the length has arrived.
        if constexpr (IND) { if (tile0 < n_tiles) request(0, tile0, 0, len); }
        else { if (tile0 * TK < l_cap) request(0, tile0, 0, l_cap); }
    }

    bf16x8 qreg[1][D / 16];
    {
        const int rho = min(l32, n_rows - 1);
        const int t = rho / group, hg = rho % group;
        const uint4* src = (const uint4*)(Qd + (((size_t)b * T_q + t) * n_q_heads + g * group + hg) * D);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) qreg[0][ks] = __builtin_bit_cast(bf16x8, src[ks * 2 + hi]);
        if constexpr (NBUF == 2) {
            // forced complete here: the compiler's wait for them covers the older request of tile 0
#pragma unroll
            for (int ks = 0; ks < D / 16; ++ks) {
                typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
                asm volatile("" :: "v"(__builtin_bit_cast(u32x4, qreg[0][ks])));
            }
        }
    }
    if constexpr (NBUF == 2 && !IND) {
        // The early request took rows past the mixed length as they are; their V values may be anything
        // (0 x NaN), so the one tile that straddles the length is fetched again with its rows clamped.
        // Loads of a wave return in order: the second copy lands on top of the first.
        if (tile0 < n_tiles && tile0 * TK + TK > len) {
            request(0, tile0, 0, len);
            wait_vmcnt<0>();
        }
    }
    f32x16 o[1][D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) o[0][db] = zero16();
    float m_run = -INFINITY, l_run = 0.f;

    auto work = [&](const uint16_t* kt, const uint16_t* vt, int rlim) {
        f32x16 s[1][1];
        qk_tile<D, 1, D, 1>(kt, qreg, l32, hi, s);
        if (rlim < TK - 1) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[0][0][r] = acc_key(0, r, hi) <= rlim ? s[0][0][r] : -INFINITY;
        }
        bf16x8 pb[1][1][2];
        softmax_tile<D / 32, 1>(s[0], c2, m_run, l_run, o[0], pb[0]);
        pv_tile<D, 1, D, 1>(vt, pb, lane, o);
    };
    if constexpr (NBUF == 1) {
        for (int i = 0; i < tiles_per_wave; ++i) {
            const int tile = tile0 + i * NW;
            if (tile >= n_tiles) break;
            const int key0 = tile * TK;
            const int rlim = min(TK - 1, len - 1 - key0);
            dma_tile_wave<D, TK>(kbase + (size_t)key0 * (D * 2), vbase + (size_t)key0 * (D * 2), Kw, Vw, lane, rlim);
            __builtin_amdgcn_s_waitcnt(0x0F70);                // vmcnt(0): the tile is in LDS
            __builtin_amdgcn_wave_barrier();
            work(Kw, Vw, rlim);
            __builtin_amdgcn_wave_barrier();
        }
    } else {
        // tile i lives in pair i & 1; tile i + 1 is requested as soon as tile i - 1 has been worked on
        if (tiles_per_wave > 1 && tile0 + NW < n_tiles) request(1, tile0 + NW, 1, len);
        for (int i = 0; i < tiles_per_wave; ++i) {
            const int tile = tile0 + i * NW;
            if (tile >= n_tiles) break;
            if (i >= 1) {
                const bool more = i + 1 < tiles_per_wave && tile + NW < n_tiles;
                if (more) request(i + 1, tile + NW, (i + 1) & 1, len);
                if (more) wait_vmcnt<2 * NL>(); else wait_vmcnt<0>();      // tile i has landed
            }
            __builtin_amdgcn_wave_barrier();
            const uint16_t* kt = Kw + (i & 1) * 2 * TILE_ELEMS;
            work(kt, kt + TILE_ELEMS, min(TK - 1, len - 1 - tile * TK));
            __builtin_amdgcn_wave_barrier();
        }
        wait_vmcnt<0>();                                       // (a wave without tiles: its early request of tile 0)
    }

    // ---- merge the waves (their tile buffers are free now): area [32 rows][D] floats per wave ----
    static_assert(32 * D * 4 <= 2 * TILE_ELEMS * 2, "merge area must fit a wave's tile pair");
    float* red = (float*)Kw;
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (l32 < n_rows) {
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                float4 v;
                v.x = o[0][db][rq * 4 + 0]; v.y = o[0][db][rq * 4 + 1];
                v.z = o[0][db][rq * 4 + 2]; v.w = o[0][db][rq * 4 + 3];
                *(float4*)(red + l32 * D + db * 32 + rq * 8 + hi * 4) = v;
            }
        if (hi == 0) { stats[wave][l32][0] = m_run; stats[wave][l32][1] = l_tot; }
    }
    __syncthreads();
    constexpr int WSTRIDE = NBUF * 2 * TILE_ELEMS / 2;         // floats between the waves' areas
    const float* red0 = (const float*)lds;
    for (int e = tid; e < n_rows * D; e += 64 * NW) {
        const int row = e / D, dd = e % D;
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, stats[w][row][0]);
        float acc = 0.f, L = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float mw = stats[w][row][0];
            const float f = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((mw - M) * c2);
            L = fmaf(f, stats[w][row][1], L);
            acc = fmaf(f, mw == -INFINITY ? 0.f : red0[w * WSTRIDE + row * D + dd], acc);
        }
        const bool empty = M == -INFINITY;
        part_o[(part_base + row) * D + dd] = empty ? 0.f : acc / L;
        if (dd == 0) part_lse[part_base + row] = empty ? -INFINITY : M * c2 + __builtin_amdgcn_logf(L);
    }
}

__device__ __forceinline__ uint16_t f32_to_bf16(float v) {
    uint32_t b = __float_as_uint(v);
    if ((b & 0x7fffffffu) > 0x7f800000u) return 0x7fc0;
    b += 0x7fffu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}

// One workgroup per query row.  Weights w_s = exp2(lse_s - max) go to LDS; the thread grid
// (split group sg, float4 column) accumulates the splits s = sg, sg + SG, ... in that order and
// the SG partial sums are added in group order; the weights are summed per wave by butterfly and
// then over the four waves: fixed summation trees, so a call gives the same bits every time.
// The first PRE partial rows of every thread are requested together with the LSEs, before the
// weights exist, so the kernel waits for memory once rather than twice (its duration is
// latency, not volume); rows of splits with weight 0 are loaded but never used.
template <int D>
__global__ __launch_bounds__(256) void decode_merge_kernel(const float* __restrict__ part_o,
                                                           const float* __restrict__ part_lse,
                                                           uint16_t* __restrict__ O, float* __restrict__ LSE,
                                                           int T_q, int n_q_heads, int n_kv_heads, int group,
                                                           int n_split) {
    constexpr int NV = D / 4;                       // float4 columns per row
    constexpr int SG = 256 / NV;                    // split groups
    constexpr int PRE = 8;                          // partial rows per thread requested up front
    extern __shared__ float sm[];
    float* w = sm;                                  // [n_split]
    float* red = sm + ((n_split + 3) & ~3);         // [SG][D]
    __shared__ float wave_max[4], wave_sum[4];
    const int n_rows = group * T_q;
    const int rho = blockIdx.x, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    const size_t base = ((size_t)b * n_kv_heads + g) * n_split;
    const int sg = tid / NV, dq = tid % NV;

    float4 pre[PRE];
#pragma unroll
    for (int i = 0; i < PRE; ++i) {
        const int s = min(sg + i * SG, n_split - 1);          // clamped: always a row of this (b, g)
        pre[i] = *(const float4*)(part_o + ((base + s) * n_rows + rho) * D + dq * 4);
    }
    float mx = -INFINITY;
    for (int s = tid; s < n_split; s += 256) {
        const float v = part_lse[(base + s) * n_rows + rho];
        w[s] = v;
        mx = fmaxf(mx, v);
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
    if ((tid & 63) == 0) wave_max[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
    float wpart = 0.f;                              // this thread's weights, then its wave's
    for (int s = tid; s < n_split; s += 256) {
        const float ws = w[s] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(w[s] - mx);
        w[s] = ws;
        wpart += ws;
    }
    for (int o = 32; o > 0; o >>= 1) wpart += __shfl_xor(wpart, o);
    if ((tid & 63) == 0) wave_sum[tid >> 6] = wpart;
    __syncthreads();

    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < PRE; ++i) {
        const int s = sg + i * SG;
        const float ws = s < n_split ? w[s] : 0.f;
        if (ws != 0.f) {
            acc.x = fmaf(ws, pre[i].x, acc.x);
            acc.y = fmaf(ws, pre[i].y, acc.y);
            acc.z = fmaf(ws, pre[i].z, acc.z);
            acc.w = fmaf(ws, pre[i].w, acc.w);
        }
    }
    for (int s = sg + PRE * SG; s < n_split; s += SG) {
        const float ws = w[s];
        if (ws != 0.f) {
            const float4 v = *(const float4*)(part_o + ((base + s) * n_rows + rho) * D + dq * 4);
            acc.x = fmaf(ws, v.x, acc.x);
            acc.y = fmaf(ws, v.y, acc.y);
            acc.z = fmaf(ws, v.z, acc.z);
            acc.w = fmaf(ws, v.w, acc.w);
        }
    }
    *(float4*)(red + sg * D + dq * 4) = acc;
    __syncthreads();
    if (tid < D) {
        float a = 0.f;
#pragma unroll
        for (int i = 0; i < SG; ++i) a += red[i * D + tid];
        const float wsum = (wave_sum[0] + wave_sum[1]) + (wave_sum[2] + wave_sum[3]);
        const int t = rho / group, hg = rho % group;
        const size_t row = ((size_t)b * T_q + t) * n_q_heads + g * group + hg;
        // an empty mixed set (every split recorded weight 0): O = 0, LSE = -inf
        const bool empty = !(wsum > 0.f);
        O[row * D + tid] = empty ? (uint16_t)0 : f32_to_bf16(a / wsum);
        if (LSE && tid == 0) LSE[row] = empty ? -INFINITY : (mx + __builtin_amdgcn_logf(wsum)) * kLn2;
    }
}

}  // namespace

template <int D, int QB>
static vxl_status run_decode(const vxl_attn_desc* d, float scale, const void* Qd, int batch, int T,
                             const void* Kmix, const void* Vmix, int l_cap, const int32_t* mix_len, void* O,
                             float* LSE, void* ws, hipStream_t s, const RowMap* rm = nullptr) {
    using C = DecodeCfg<D, QB>;
    const DecodePlan p = decode_plan(d, batch, T, l_cap, rm == nullptr);
    float* part_o = (float*)((char*)ws + p.part_o);
    float* part_lse = (float*)((char*)ws + p.part_ml);
    const int group = d->n_q_heads / d->n_kv_heads;
    const int n_rows = group * T;
    const int n_rtile = (n_rows + C::RT - 1) / C::RT;
    static PerDeviceOnce attr;
    const vxl_status ast = attr.run([] {
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)decode_split_kernel<D, QB, false>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)decode_split_kernel<D, QB, true>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        return VXL_OK;
    });
    if (ast != VXL_OK) return ast;
    if (rm)
        hipLaunchKernelGGL((decode_split_kernel<D, QB, true>), dim3(p.n_split, n_rtile * d->n_kv_heads, batch),
                           dim3(256), C::LDS_BYTES, s, (const uint16_t*)Qd, (const uint16_t*)Kmix,
                           (const uint16_t*)Vmix, mix_len, part_o, part_lse, T, d->n_q_heads, d->n_kv_heads, group,
                           l_cap, n_rtile, p.split_len, scale, *rm);
    else
        hipLaunchKernelGGL((decode_split_kernel<D, QB, false>), dim3(p.n_split, n_rtile * d->n_kv_heads, batch),
                           dim3(256), C::LDS_BYTES, s, (const uint16_t*)Qd, (const uint16_t*)Kmix,
                           (const uint16_t*)Vmix, mix_len, part_o, part_lse, T, d->n_q_heads, d->n_kv_heads, group,
                           l_cap, n_rtile, p.split_len, scale, RowMap{});
    VXL_HIP_TRY(hipGetLastError());
    const size_t merge_lds = (size_t)(((p.n_split + 3) & ~3) + 256 / (D / 4) * D) * sizeof(float);
    hipLaunchKernelGGL((decode_merge_kernel<D>), dim3(n_rows, d->n_kv_heads, batch), dim3(256), merge_lds, s,
                       part_o, part_lse, (uint16_t*)O, LSE, T, d->n_q_heads, d->n_kv_heads, group, p.n_split);
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

template <int D>
static vxl_status run_decode_ring(const vxl_attn_desc* d, float scale, const void* Qd, int batch, int T,
                                  const void* Kmix, const void* Vmix, int l_cap, const int32_t* mix_len, void* O,
                                  float* LSE, void* ws, hipStream_t s, const RowMap* rm = nullptr) {
    using C = DecodeRingCfg<D, 4>;
    const DecodePlan p = decode_plan(d, batch, T, l_cap, rm == nullptr);
    float* part_o = (float*)((char*)ws + p.part_o);
    float* part_lse = (float*)((char*)ws + p.part_ml);
    const int group = d->n_q_heads / d->n_kv_heads;
    const int n_rows = group * T;
    const int n_rtile = (n_rows + C::RT - 1) / C::RT;
    static PerDeviceOnce attr;
    const vxl_status ast = attr.run([] {
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)decode_ring_kernel<D, 4, false>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)decode_ring_kernel<D, 4, true>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        return VXL_OK;
    });
    if (ast != VXL_OK) return ast;
    if (rm)
        hipLaunchKernelGGL((decode_ring_kernel<D, 4, true>), dim3(p.n_split, n_rtile * d->n_kv_heads, batch),
                           dim3(512), C::LDS_BYTES, s, (const uint16_t*)Qd, (const uint16_t*)Kmix,
                           (const uint16_t*)Vmix, mix_len, part_o, part_lse, T, d->n_q_heads, d->n_kv_heads, group,
                           l_cap, n_rtile, p.split_len, scale, *rm);
    else
        hipLaunchKernelGGL((decode_ring_kernel<D, 4, false>), dim3(p.n_split, n_rtile * d->n_kv_heads, batch),
                           dim3(512), C::LDS_BYTES, s, (const uint16_t*)Qd, (const uint16_t*)Kmix,
                           (const uint16_t*)Vmix, mix_len, part_o, part_lse, T, d->n_q_heads, d->n_kv_heads, group,
                           l_cap, n_rtile, p.split_len, scale, RowMap{});
    VXL_HIP_TRY(hipGetLastError());
    const size_t merge_lds = (size_t)(((p.n_split + 3) & ~3) + 256 / (D / 4) * D) * sizeof(float);
    hipLaunchKernelGGL((decode_merge_kernel<D>), dim3(n_rows, d->n_kv_heads, batch), dim3(256), merge_lds, s,
                       part_o, part_lse, (uint16_t*)O, LSE, T, d->n_q_heads, d->n_kv_heads, group, p.n_split);
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

template <int D>
static vxl_status run_decode_wave(const vxl_attn_desc* d, float scale, const void* Qd, int batch, int T,
                                  const void* Kmix, const void* Vmix, int l_cap, const int32_t* mix_len, void* O,
                                  float* LSE, void* ws, hipStream_t s, const RowMap* rm = nullptr) {
    const DecodePlan p = decode_plan(d, batch, T, l_cap, rm == nullptr);
    float* part_o = (float*)((char*)ws + p.part_o);
    float* part_lse = (float*)((char*)ws + p.part_ml);
    const int group = d->n_q_heads / d->n_kv_heads;
    const int n_rows = group * T;
    constexpr int lds_bytes = 8 * 2 * kStepTile * D * 2;      // 8 tile pairs in either form
    static PerDeviceOnce attr;
    const vxl_status ast = attr.run([] {
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)decode_wave_kernel<D, 8, 1>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)decode_wave_kernel<D, 4, 2>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        VXL_HIP_TRY(hipFuncSetAttribute((const void*)decode_wave_kernel<D, 4, 2, true>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes));
        return VXL_OK;
    });
    if (ast != VXL_OK) return ast;
    if (rm) {
        // (the plan of the in-place form always has 4 waves; the row map of a wave's tiles must fit its LDS area)
        if (p.split_len / (4 * kStepTile) > kMaxStepTpw) return VXL_ERR_UNSUPPORTED;
        hipLaunchKernelGGL((decode_wave_kernel<D, 4, 2, true>), dim3(p.n_split, d->n_kv_heads, batch), dim3(256),
                           lds_bytes, s, (const uint16_t*)Qd, (const uint16_t*)Kmix, (const uint16_t*)Vmix,
                           mix_len, part_o, part_lse, T, d->n_q_heads, d->n_kv_heads, group, l_cap,
                           p.split_len / (4 * kStepTile), scale, *rm);
    } else if (p.step_waves == 8)
        hipLaunchKernelGGL((decode_wave_kernel<D, 8, 1>), dim3(p.n_split, d->n_kv_heads, batch), dim3(512),
                           lds_bytes, s, (const uint16_t*)Qd, (const uint16_t*)Kmix, (const uint16_t*)Vmix,
                           mix_len, part_o, part_lse, T, d->n_q_heads, d->n_kv_heads, group, l_cap,
                           p.split_len / (8 * kStepTile), scale, RowMap{});
    else
        hipLaunchKernelGGL((decode_wave_kernel<D, 4, 2>), dim3(p.n_split, d->n_kv_heads, batch), dim3(256),
                           lds_bytes, s, (const uint16_t*)Qd, (const uint16_t*)Kmix, (const uint16_t*)Vmix,
                           mix_len, part_o, part_lse, T, d->n_q_heads, d->n_kv_heads, group, l_cap,
                           p.split_len / (4 * kStepTile), scale, RowMap{});
    VXL_HIP_TRY(hipGetLastError());
    const size_t merge_lds = (size_t)(((p.n_split + 3) & ~3) + 256 / (D / 4) * D) * sizeof(float);
    hipLaunchKernelGGL((decode_merge_kernel<D>), dim3(n_rows, d->n_kv_heads, batch), dim3(256), merge_lds, s,
                       part_o, part_lse, (uint16_t*)O, LSE, T, d->n_q_heads, d->n_kv_heads, group, p.n_split);
    VXL_HIP_TRY(hipGetLastError());
    return VXL_OK;
}

// Scratch of the entry point that allocates nothing: one array per device, held until the process
// ends.  In host code the name below is only a stand-in for the symbol; the device address is
// asked for once per device (with that device current) and kept.
static __device__ __align__(256) unsigned char scratch[VXL_STATIC_SCRATCH_BYTES];

vxl_status decode_static_scratch(void** ptr) {
    static std::mutex mu;
    static void* addr[kMaxDevices] = {};
    int dev = 0;
    VXL_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return VXL_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void* p = nullptr;
        VXL_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return VXL_ERR_HIP;
        addr[dev] = p;
    }
    *ptr = addr[dev];
    return VXL_OK;
}

vxl_status launch_decode_bf16(const vxl_attn_desc* d, float scale, const void* Qd, int batch, int T,
                              const void* Kmix, const void* Vmix, int l_cap, const int32_t* mix_len, void* O,
                              float* LSE, void* ws, hipStream_t s) {
    const int n_rows = (d->n_q_heads / d->n_kv_heads) * T;
    if (n_rows <= kRowBlock)
        return d->head_dim == 128
                   ? run_decode_wave<128>(d, scale, Qd, batch, T, Kmix, Vmix, l_cap, mix_len, O, LSE, ws, s)
                   : run_decode_wave<64>(d, scale, Qd, batch, T, Kmix, Vmix, l_cap, mix_len, O, LSE, ws, s);
    const bool big = decode_plan(d, batch, T, l_cap).use_ring != 0;
    if (d->head_dim == 128)
        return big ? run_decode_ring<128>(d, scale, Qd, batch, T, Kmix, Vmix, l_cap, mix_len, O, LSE, ws, s)
                   : run_decode<128, 1>(d, scale, Qd, batch, T, Kmix, Vmix, l_cap, mix_len, O, LSE, ws, s);
    return big ? run_decode_ring<64>(d, scale, Qd, batch, T, Kmix, Vmix, l_cap, mix_len, O, LSE, ws, s)
               : run_decode<64, 1>(d, scale, Qd, batch, T, Kmix, Vmix, l_cap, mix_len, O, LSE, ws, s);
}

// In-place form: K / V are the dense tensors of the layer, rows reached through src_idx.
vxl_status launch_decode_bf16_inplace(const vxl_layout* L, const vxl_attn_desc* d, float scale, const void* Qd,
                                      int batch, int T, const void* K, const void* V, const void* Ksp,
                                      const void* Vsp, const int32_t* src_idx, int l_cap, const int32_t* mix_len,
                                      void* O, float* LSE, void* ws, hipStream_t s) {
    const TokStrides ts = tok_strides(d, L->n_tokens);
    const RowMap rm{src_idx, (const uint16_t*)Ksp, (const uint16_t*)Vsp, ts.kh, ts.kt, L->s_total};
    const int n_rows = (d->n_q_heads / d->n_kv_heads) * T;
    if (n_rows <= kRowBlock)
        return d->head_dim == 128
                   ? run_decode_wave<128>(d, scale, Qd, batch, T, K, V, l_cap, mix_len, O, LSE, ws, s, &rm)
                   : run_decode_wave<64>(d, scale, Qd, batch, T, K, V, l_cap, mix_len, O, LSE, ws, s, &rm);
    const bool big = decode_plan(d, batch, T, l_cap, false).use_ring != 0;
    if (d->head_dim == 128)
        return big ? run_decode_ring<128>(d, scale, Qd, batch, T, K, V, l_cap, mix_len, O, LSE, ws, s, &rm)
                   : run_decode<128, 1>(d, scale, Qd, batch, T, K, V, l_cap, mix_len, O, LSE, ws, s, &rm);
    return big ? run_decode_ring<64>(d, scale, Qd, batch, T, K, V, l_cap, mix_len, O, LSE, ws, s, &rm)
               : run_decode<64, 1>(d, scale, Qd, batch, T, K, V, l_cap, mix_len, O, LSE, ws, s, &rm);
}

}  // namespace vxl
