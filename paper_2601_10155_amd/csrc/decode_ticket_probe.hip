// Measurement aid, not part of the product path: lookat_attend_decode on a FLAT launch geometry with the
// merge of the pieces done inside the kernel (a ticket per (b,h) unit) instead of by a second launch.
// It computes the same result (paper Algorithm 1 after the table build) and exists so that the cost of an
// in-kernel merge on this chip can be measured against the two-launch path of decode.hip with committed
// code.  Measured on MI355X: publication and merge are three dependent round trips to memory (write-through
// stores, a device-scope ticket, cache-bypassing loads); under the load of the value stream they cost about
// 1 us at batch 32 x 12 heads x 1024 keys even when a wavefront of its own does them behind the streaming,
// and about 3.5 us MORE than the second launch at 32 (b,h) x 32768 keys.
#include "decode_common.h"
#include "lookat_probe.h"

namespace lookat {

// ---------------------------------------------------------------------------------------------
// Flat launch geometry with an in-kernel merge.
//
// The key tiles (64 keys) of all (b,h) units form one flat index space: unit u owns the flat tiles
// [u * tpu, (u + 1) * tpu)  (tpu = tiles per unit, padded where a caller asks for a fixed number of
// ranges per unit).  Workgroup share sigma covers the flat tiles [sigma * share, (sigma + 1) * share),
// i.e. a tail of one unit, whole units, a head of another: at most kFlatPieces pieces.  A unit that
// several workgroups cover is merged in-kernel: every piece publishes its (o, max, sum) in the
// workspace and takes a ticket from the unit's counter; the workgroup that draws the last ticket
// reads all pieces of the unit, merges them (the exact merge of the online softmax) and writes `out`,
// then puts the counter back to zero.  No second launch, and the shares are equal whatever B*H is.
// ---------------------------------------------------------------------------------------------
constexpr int kFlatWaves = 8;      // one workgroup of 512 threads per compute unit streams best (measured)
constexpr int kFlatPieces = 3;     // share <= 2 units: tail + whole + head

// n / d for a kernel-uniform divisor, from numbers the host prepares (Granlund-Montgomery, exact for
// every 32-bit n): q = (t + ((n - t) >> sh1)) >> sh2 with t = mulhi(magic, n).
struct FastDiv {
    uint32_t magic;
    uint32_t sh1, sh2;
};
static FastDiv fastdiv_of(uint32_t d)
{
    FastDiv f;
    if (d <= 1) {
        f.magic = 0;
        f.sh1 = 0;
        f.sh2 = 0;
        return f;
    }
    uint32_t l = 0;
    while ((1ull << l) < d)
        ++l;   // l = ceil(log2 d)
    f.magic = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    f.sh1 = 1;
    f.sh2 = l - 1;
    return f;
}
__device__ __forceinline__ uint32_t fastdiv(uint32_t n, uint32_t magic, uint32_t sh1, uint32_t sh2)
{
    const uint32_t t = __umulhi(magic, n);
    return (t + ((n - t) >> sh1)) >> sh2;
}

struct FlatLate {
    float *part;           // [BH][slots][d_k + 2]
    unsigned *tickets;     // [BH], zero between launches
    float *out;            // [BH][d_k]
    float *scores_out;     // [BH][L] or nullptr
    int slots;             // pieces a unit can have (size of its row in `part`)
    float scale_log2e;
};

// What a piece's finishing wavefront does with the piece's result.  Lane l holds the unnormalised output
// coordinates o[x] = o_{x*64 + l}; mx and zz (max and sum of the piece) are wavefront-uniform.  A unit covered
// by one piece is normalised and written out; otherwise the piece is published and a ticket drawn, and the
// last ticket merges.  Called by all 64 lanes of ONE wavefront.
template <int DK>
__device__ __forceinline__ void finish_piece(const FlatLate &late, const float (&o)[(DK + kWave - 1) / kWave], float mx,
                                             float zz, uint32_t u, uint32_t slot, uint32_t pieces, int lane)
{
    constexpr int E = DK + 2;
    constexpr int X = (DK + kWave - 1) / kWave;
    if (pieces == 1) {
#pragma unroll
        for (int x = 0; x < X; ++x)
            if (x * kWave + lane < DK)
                late.out[(int64_t)u * DK + x * kWave + lane] = o[x] / zz;
        return;
    }
    // The pieces of a unit may run on different dies, whose L2 caches are not coherent with each other.
    // Everything exchanged here therefore moves with device-scope relaxed atomic accesses (stores that
    // write through to memory, loads that bypass the caches, one read-modify-write at memory for the
    // ticket), ordered by waiting for the stores before the ticket is drawn; a device-scope FENCE would
    // write back and invalidate the whole L2 of the die and was measured at 3 to 20 times the kernel.
    float *mine = late.part + ((int64_t)u * late.slots + slot) * E;
#pragma unroll
    for (int x = 0; x < X; ++x)
        if (x * kWave + lane < DK)
            __hip_atomic_store(mine + x * kWave + lane, o[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (lane == 0) {
        __hip_atomic_store(mine + DK, mx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(mine + DK + 1, zz, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // compiler: nothing above sinks below
    __builtin_amdgcn_s_waitcnt(0);                           // hardware: the wavefront's stores have been performed
    unsigned ticket = 0;
    if (lane == 0)
        ticket = __hip_atomic_fetch_add(late.tickets + u, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    if (ticket + 1 != pieces)
        return;
    // Last arriver: every other piece stored before it drew its ticket.
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");   // compiler: nothing below rises above
    const float *all = late.part + (int64_t)u * late.slots * E;
    float gmx = -INFINITY;
    for (uint32_t s = 0; s < pieces; ++s)
        gmx = fmaxf(gmx, __hip_atomic_load(all + s * E + DK, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    const float m_use = (gmx == -INFINITY) ? 0.f : gmx;
    float gz = 0.f;
    float go[X];
#pragma unroll
    for (int x = 0; x < X; ++x)
        go[x] = 0.f;
    for (uint32_t s = 0; s < pieces; ++s) {
        const float w = fast_exp2(__hip_atomic_load(all + s * E + DK, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - m_use);
        gz = fmaf(w, __hip_atomic_load(all + s * E + DK + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), gz);
#pragma unroll
        for (int x = 0; x < X; ++x)
            if (x * kWave + lane < DK)
                go[x] = fmaf(w, __hip_atomic_load(all + s * E + x * kWave + lane, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT),
                             go[x]);
    }
#pragma unroll
    for (int x = 0; x < X; ++x)
        if (x * kWave + lane < DK)
            late.out[(int64_t)u * DK + x * kWave + lane] = go[x] / gz;
    if (lane == 0)   // the counter goes back to zero for the next launch (ordered by the kernel boundary)
        __hip_atomic_store(late.tickets + u, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The 14 dwords that arrive in scalar registers at wave launch (see DecodeLate): everything a wavefront
// needs to request its first tile.  p_H_sh: heads in bits 0..15, the shift pairs of the two divisors
// (tiles per unit: bits 16..21, heads: bits 22..27).
// (An even number of dwords ahead of the pointers: a padding dword would push the last one out of the 14.)
#define LOOKAT_FLAT_HEAD_PARAMS                                                                                \
    uint32_t p_nflat, uint32_t p_share, uint32_t p_magic_tu, uint32_t p_H_sh, const void *p_table,            \
        const uint8_t *p_codes, const __half *p_values, uint32_t p_code_stride, uint32_t p_value_stride,      \
        uint32_t p_L, uint32_t p_magic_H

// One 64-key tile, tables given (G = 1): scores one key per lane, updates the wavefront's running
// max / sum and accumulates the weighted value rows.  klim: keys >= klim are masked.
template <int DK, int M, int CH>
__device__ __forceinline__ void flat_consume(SoftmaxState<1> &st, const KeyCodes<M> &kc, v4u (&v)[CH], const float *lut_s,
                                             __amdgpu_buffer_rsrc_t rv, float *scores_u, float scale_log2e,
                                             uint32_t kb, uint32_t klim, uint32_t kofs, int lane)
{
    constexpr int LPR = DK / 8;
    constexpr int NLD = LPR;
    const uint32_t key = kb + kofs;
    const float raw = kc.score(lut_s);
    float s = -INFINITY;
    if (key < klim) {
        if (scores_u)
            scores_u[key] = raw;
        s = raw * scale_log2e;
    }
    const float m_new = fmaxf(st.m_run[0], wave_max(s));
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float corr = fast_exp2(st.m_run[0] - m_use);
    const float p = fast_exp2(s - m_use);
    st.z[0] = st.z[0] * corr + p;
#pragma unroll
    for (int d = 0; d < 8; ++d)
        st.acc[0][d] *= corr;
    st.m_run[0] = m_new;
#pragma unroll
    for (int c0 = 0; c0 < NLD; c0 += CH) {
        fma_rows<LPR, CH>(st.acc[0], p, v, c0);
        if (c0 + CH < NLD)
            load_rows<DK, CH>(v, rv, kb, c0 + CH, lane);
    }
}

// lookat_attend_decode on the flat geometry.  DK in {32, 64, 128, 256}, M in {2, 4, 8, 16}.
// WAVES wavefronts stream; with SVC = 1 one more wavefront streams nothing and does the finishing of every
// piece (the fold over the wavefronts' results, publication, ticket, merge, output), so that no streaming
// wavefront stalls for the round trips of a publication while it has tiles left.
template <int DK, int M, int WAVES, int SVC>
__global__ __launch_bounds__((WAVES + SVC) * kWave, (WAVES == 8 ? 2 : 1)) void decode_flat_kernel(LOOKAT_FLAT_HEAD_PARAMS,
                                                                                                  const FlatLate late)
{
    constexpr int NT = (WAVES + SVC) * kWave;
    constexpr int LPR = DK / 8;
    constexpr int RPL = kWave / LPR;
    constexpr int NLD = kTile / RPL;
    constexpr int CH = NLD < 8 ? NLD : 8;
    constexpr int E = DK + 2;
    constexpr int kTableVec = M * (kCentroids / 4);                  // 16-byte pieces of one unit's tables
    constexpr int kLutRegs = (kTableVec + NT - 1) / NT;              // per thread and piece

    extern __shared__ __align__(16) float smem[];
    float *lut_s = smem;                                             // [kFlatPieces][M][256]
    float *red_s = smem + kFlatPieces * M * kCentroids;              // [kFlatPieces][WAVES][E]
    unsigned *done_s = reinterpret_cast<unsigned *>(red_s + kFlatPieces * WAVES * E);   // [kFlatPieces] wavefronts that have folded piece i

    // ---- this workgroup's share of the flat tile space: as little scalar arithmetic as possible ahead of the
    //      first requests (every hundred instructions here add 0.2 us to a 10 us kernel) ----
    const uint32_t sigma = blockIdx.x;
    const uint32_t p_tpu = (p_L + kTile - 1) / kTile;               // tiles per unit
    const uint32_t f0 = sigma * p_share;
    if (f0 >= p_nflat)
        return;
    const uint32_t len = (p_nflat - f0 < p_share) ? p_nflat - f0 : p_share;
    const uint32_t u0 = fastdiv(f0, p_magic_tu, (p_H_sh >> 16) & 1u, (p_H_sh >> 17) & 31u);
    const uint32_t ft0 = f0 - u0 * p_tpu;                           // first tile of the share within unit u0
    const uint32_t fe = ft0 + len;                                  // end of the share, in tiles from the start of unit u0
    const int np = 1 + (fe > p_tpu ? 1 : 0) + (fe > 2 * p_tpu ? 1 : 0);   // pieces: 1 .. kFlatPieces (the host's plan guarantees it)
    const uint32_t ftl = fe - (uint32_t)(np - 1) * p_tpu;           // end tile of the last piece within its unit
    const uint32_t tiles_valid = p_tpu;

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int sub = lane % LPR;
    const int rowin = lane / LPR;
    const uint32_t kofs = (uint32_t)(RPL * sub + rowin);

    // piece p: unit u0 + p, tiles [t0, t1) of it
#define LOOKAT_PIECE_T0(p) ((p) == 0 ? ft0 : 0u)
#define LOOKAT_PIECE_T1(p) ((p) == np - 1 ? ftl : p_tpu)

    // ---- requests, in the order they are needed: tables of every piece, codes and rows of the first tile ----
    // Through buffer descriptors whose size says what exists: a piece this workgroup does not have gets a
    // descriptor of no bytes, threads beyond the table fall outside it; both read zero without a memory
    // access and without a branch.
    v4f lut_r[kFlatPieces][kLutRegs];   // (a plain vector type: arrays of float4 structs end up in scratch memory)
#pragma unroll
    for (int p = 0; p < kFlatPieces; ++p) {
        const __amdgpu_buffer_rsrc_t rt = make_rsrc(static_cast<const char *>(p_table) + (int64_t)(u0 + p) * (kTableVec * 16),
                                                   p < np ? (uint32_t)(kTableVec * 16) : 0u);
#pragma unroll
        for (int x = 0; x < kLutRegs; ++x) {
            const v4u t = __builtin_amdgcn_raw_buffer_load_b128(rt, (uint32_t)(tid + x * NT) * 16u, 0, 0);
            lut_r[p][x] = __builtin_bit_cast(v4f, t);
        }
    }
    KeyCodes<M> kc;
    v4u v[CH];
    __amdgpu_buffer_rsrc_t rv, rc;
    uint32_t klim = 0;
    // Descriptors of a piece's unit and the request of this wavefront's first tile of the piece (if it has
    // one).  (A macro: a lambda that captures the register arrays sends them through scratch memory.)
    bool have;
#define LOOKAT_OPEN_PIECE(p)                                                                                   \
    {                                                                                                          \
        const uint32_t u_ = u0 + (uint32_t)(p);                                                                \
        const uint32_t t1_ = LOOKAT_PIECE_T1(p);                                                               \
        const uint32_t tv_ = t1_ < tiles_valid ? t1_ : tiles_valid;                                            \
        klim = (tv_ * kTile < p_L) ? tv_ * kTile : p_L;                                                        \
        rv = make_rsrc(p_values + (int64_t)u_ * p_value_stride, klim * (uint32_t)(DK * 2));                    \
        rc = make_rsrc(p_codes + (int64_t)u_ * p_code_stride, klim * (uint32_t)M);                             \
        const uint32_t t_ = LOOKAT_PIECE_T0(p) + (uint32_t)wave;                                               \
        have = t_ < tv_;                                                                                       \
        if (have) {                                                                                            \
            kc.load(rc, (t_ * kTile + kofs) * M);                                                              \
            __builtin_amdgcn_sched_barrier(0); /* request order = need order: codes before value rows */       \
            load_rows<DK, CH>(v, rv, t_ * kTile, 0, lane);                                                     \
        }                                                                                                      \
    }
    // Processing order: pieces of units that other workgroups share come first, so that their publication
    // and merge (three round trips to memory) hide behind the streaming of the rest.
    // (a whole first piece followed by a partial last one: the last goes first; otherwise the natural order
    // with a partial last piece ahead of a whole middle one)
    const bool last_first = ft0 == 0u && np > 1 && ftl != p_tpu;
    int ord[kFlatPieces];
    ord[0] = last_first ? np - 1 : 0;
    ord[1] = last_first ? 0 : ((np == 3 && ftl != p_tpu) ? 2 : 1);
    ord[2] = 3 - ord[0] - ord[1];
    const bool streams = !SVC || wave < WAVES;
    const bool finishes = SVC ? wave == WAVES : wave == 0;
    have = false;
    if (streams)
        LOOKAT_OPEN_PIECE(ord[0])
    if (SVC && tid < kFlatPieces)
        done_s[tid] = 0u;
    {
        v4f *s4 = reinterpret_cast<v4f *>(lut_s);
#pragma unroll
        for (int p = 0; p < kFlatPieces; ++p) {
            if (p < np) {
#pragma unroll
                for (int x = 0; x < kLutRegs; ++x)
                    if ((x + 1) * NT <= kTableVec || tid + x * NT < kTableVec)
                        s4[p * kTableVec + tid + x * NT] = lut_r[p][x];
            }
        }
    }
    __syncthreads();   // tables in LDS; the tile stays in flight

#pragma unroll
    for (int i = 0; i < kFlatPieces; ++i) {
        if (i >= np)
            break;
        const int p = ord[i];
        const uint32_t u = u0 + (uint32_t)p;
        const uint32_t t0 = LOOKAT_PIECE_T0(p), t1 = LOOKAT_PIECE_T1(p);
        const uint32_t tv = t1 < tiles_valid ? t1 : tiles_valid;
        float *scores_u = late.scores_out ? late.scores_out + (int64_t)u * p_L : nullptr;
        const float *lut_p = lut_s + p * (M * kCentroids);
        SoftmaxState<1> st;
        if (have) {
            uint32_t t = t0 + (uint32_t)wave;
            flat_consume<DK, M, CH>(st, kc, v, lut_p, rv, scores_u, late.scale_log2e, t * kTile, klim, kofs, lane);
            for (t += WAVES; t < tv; t += WAVES) {
                kc.load(rc, (t * kTile + kofs) * M);
                __builtin_amdgcn_sched_barrier(0);
                load_rows<DK, CH>(v, rv, t * kTile, 0, lane);
                flat_consume<DK, M, CH>(st, kc, v, lut_p, rv, scores_u, late.scale_log2e, t * kTile, klim, kofs, lane);
            }
        }
        if (streams) {
            // the next piece's first tile travels while this piece is folded and finished
            have = false;
            if (i + 1 < np)
                LOOKAT_OPEN_PIECE(ord[i + 1])

            // ---- fold the lanes of the wavefront, then the wavefronts (through LDS) ----
#pragma unroll
            for (int d = 0; d < 8; ++d)
                st.acc[0][d] = sum_over_lane_classes<LPR>(st.acc[0][d]);
            st.z[0] = wave_sum(st.z[0]);
            float *mine = red_s + (i * WAVES + wave) * E;
            if (lane < LPR) {
#pragma unroll
                for (int d = 0; d < 8; ++d)
                    mine[sub * 8 + d] = st.acc[0][d];
            }
            if (lane == 0) {
                mine[DK] = st.m_run[0];
                mine[DK + 1] = st.z[0];
            }
        }
        // With a finishing wavefront of its own nobody waits at a barrier: the streaming wavefronts count
        // themselves off (after their results are in LDS) and go on; the finisher waits for the count.
        if constexpr (SVC) {
            if (streams) {
                if (lane == 0)
                    __hip_atomic_fetch_add(done_s + i, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            } else {
                while (__hip_atomic_load(done_s + i, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < (unsigned)WAVES)
                    __builtin_amdgcn_s_sleep(4);
            }
        } else {
            __syncthreads();
        }
        if (finishes) {
            const float *rs = red_s + i * WAVES * E;
            float mx = -INFINITY;
#pragma unroll
            for (int w = 0; w < WAVES; ++w)
                mx = fmaxf(mx, rs[w * E + DK]);
            const float m_use = (mx == -INFINITY) ? 0.f : mx;
            float wgt[WAVES];
            float zz = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) {
                wgt[w] = fast_exp2(rs[w * E + DK] - m_use);
                zz = fmaf(wgt[w], rs[w * E + DK + 1], zz);
            }
            float o[(DK + kWave - 1) / kWave];
#pragma unroll
            for (int x = 0; x < (DK + kWave - 1) / kWave; ++x) {
                o[x] = 0.f;
                if (x * kWave + lane < DK) {
#pragma unroll
                    for (int w = 0; w < WAVES; ++w)
                        o[x] = fmaf(wgt[w], rs[w * E + x * kWave + lane], o[x]);
                }
            }
            // pieces of this unit: the shares that overlap [u * tpu, (u + 1) * tpu)
            uint32_t pieces = 1, slot = 0;
            if (t0 != 0 || t1 != p_tpu) {
                const uint32_t first = (u * p_tpu) / p_share;
                pieces = ((u + 1) * p_tpu - 1) / p_share - first + 1;
                slot = sigma - first;
            }
            finish_piece<DK>(late, o, mx, zz, u, slot, pieces, lane);
        }
    }
}

#undef LOOKAT_OPEN_PIECE
#undef LOOKAT_PIECE_T0
#undef LOOKAT_PIECE_T1

// Shapes the flat-geometry kernel handles.
static bool flat_shape(const lookat_shape *s)
{
    return (s->d_k == 32 || s->d_k == 64 || s->d_k == 128 || s->d_k == 256) && (s->m == 2 || s->m == 4 || s->m == 8 || s->m == 16);
}

// Launch geometry of the flat kernels (see decode_flat_kernel): tiles per unit, tiles per workgroup,
// workgroups, and the most pieces a unit can be cut into.
struct FlatPlan {
    int64_t tpu, share, shares, slots;
};
static FlatPlan plan_flat(int64_t BH, int64_t L, int32_t num_splits)
{
    constexpr int64_t kUnits = 256;              // compute units of the chip
    constexpr int64_t kMinRange = 2048 / kTile;  // auto: no range shorter than 2048 keys (measured, see auto_splits)
    FlatPlan g;
    const int64_t tu = (L + kTile - 1) / kTile;
    const int64_t total = BH * tu;
    int64_t share;
    if (num_splits >= 1) {   // the caller's count: shares of ceil(tiles / count) tiles
        share = (tu + num_splits - 1) / num_splits;
    } else {
        share = (total + kUnits - 1) / kUnits;   // equal shares, one workgroup per compute unit
        if (share >= tu) {
            if (share * 4 < tu * 5)
                share = tu;                  // under 1.25 units per workgroup: whole units, nothing to merge
            if (share > 2 * tu)
                share = 2 * tu;              // at most tail + whole unit + head (kFlatPieces)
        } else {
            if (share < kMinRange)
                share = kMinRange;
            if (share > tu)
                share = tu;
        }
    }
    g.tpu = tu;
    g.share = share;
    g.shares = (total + share - 1) / share;
    g.slots = (tu % share == 0) ? tu / share : (tu - 1) / share + 2;   // most pieces a unit can be cut into
    return g;
}
// Wavefronts per workgroup: 16 where a workgroup streams long ranges of a unit (at least 32 tiles each; measured at
// 32 (b,h) x 32768 keys), 8 otherwise; d_k = 256 keeps 8 (a 16-wavefront workgroup must fit 128 registers).
static int flat_waves(int d_k, const FlatPlan &g)
{
    return (d_k <= 128 && g.share >= 32 && g.share <= g.tpu) ? 16 : kFlatWaves;
}
// Workspace of the flat kernels: one ticket counter per unit first (a fixed place whatever the geometry),
// then the published pieces [BH][slots][d_k + 2].
static size_t flat_ticket_bytes(int64_t BH) { return ((size_t)BH * sizeof(unsigned) + 255) / 256 * 256; }
static size_t flat_part_bytes(int64_t BH, int d_k, const FlatPlan &g)
{
    return g.slots <= 1 ? 0 : (size_t)BH * g.slots * (d_k + 2) * sizeof(float);
}
static size_t flat_workspace_bytes(int64_t BH, int d_k, const FlatPlan &g)
{
    return g.slots <= 1 ? 0 : flat_ticket_bytes(BH) + flat_part_bytes(BH, d_k, g);
}

template <int DK, int WAVES, int SVC>
static void launch_flat(int m, dim3 grid, size_t lds, hipStream_t st, uint32_t nflat, uint32_t share, uint32_t magic_tu,
                        uint32_t H_sh, const float *lut, const uint8_t *codes, const __half *values, uint32_t cs,
                        uint32_t vs, uint32_t L, const FlatLate &late)
{
#define LOOKAT_FLAT_CASE(M_)                                                                                       \
    case M_:                                                                                                       \
        hipLaunchKernelGGL((decode_flat_kernel<DK, M_, WAVES, SVC>), grid, dim3((WAVES + SVC) * kWave), lds, st, nflat, \
                           share, magic_tu, H_sh, static_cast<const void *>(lut), codes, values, cs, vs, L, 0u, late); \
        break;
    switch (m) {
        LOOKAT_FLAT_CASE(2)
        LOOKAT_FLAT_CASE(4)
        LOOKAT_FLAT_CASE(8)
        LOOKAT_FLAT_CASE(16)
    }
#undef LOOKAT_FLAT_CASE
}


}  // namespace lookat

extern "C" size_t lookat_probe_attend_decode_ticket_workspace_bytes(const lookat_shape *shape, int64_t L, int32_t num_splits)
{
    using namespace lookat;
    clear_error();
    if (check_shape(shape) != LOOKAT_OK || !flat_shape(shape) || L <= 0 || num_splits < 0)
        return 0;
    const int64_t BH = (int64_t)shape->B * shape->H;
    return flat_workspace_bytes(BH, shape->d_k, plan_flat(BH, L, num_splits));
}

extern "C" int lookat_probe_attend_decode_ticket(const lookat_shape *shape, int64_t L, const float *lut, const uint8_t *codes,
                                                 int64_t code_stride_bh, const void *values, int64_t value_stride_bh,
                                                 float scale, int32_t num_splits, void *workspace, size_t workspace_bytes,
                                                 float *out, float *scores_out, int32_t *pieces_per_unit, void *stream)
{
    using namespace lookat;
    clear_error();
    if (int rc = check_shape(shape))
        return rc;
    if (!flat_shape(shape))
        return fail(LOOKAT_ERR_UNSUPPORTED, "the ticket-merge probe handles d_k in {32,64,128,256} with m in {2,4,8,16}");
    if (L <= 0)
        return fail(LOOKAT_ERR_SHAPE, "L=%lld must be positive", (long long)L);
    if (num_splits < 0 || num_splits > 65535)
        return fail(LOOKAT_ERR_SHAPE, "num_splits=%d out of range [0,65535]", num_splits);
    if (!lut || !codes || !values || !out)
        return fail(LOOKAT_ERR_NULL, "lut, codes, values and out must be non-NULL");
    if (code_stride_bh < L * shape->m || value_stride_bh < L * shape->d_k)
        return fail(LOOKAT_ERR_SHAPE, "code_stride_bh=%lld / value_stride_bh=%lld smaller than one (b,h) slab",
                    (long long)code_stride_bh, (long long)value_stride_bh);
    if (!aligned16(lut) || !aligned16(values) || !aligned16(out) || ((value_stride_bh * 2) % 16))
        return fail(LOOKAT_ERR_ALIGN, "lut, values, out and value_stride_bh must be 16-byte aligned");
    if ((reinterpret_cast<uintptr_t>(codes) % shape->m) || (code_stride_bh % shape->m))
        return fail(LOOKAT_ERR_ALIGN, "codes and code_stride_bh must be multiples of m=%d bytes", shape->m);
    if (scores_out && (reinterpret_cast<uintptr_t>(scores_out) & 3u))
        return fail(LOOKAT_ERR_ALIGN, "scores_out must be 4-byte aligned");
    if (code_stride_bh > 0xffffffffLL || value_stride_bh > 0xffffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "(b,h) strides must stay below 2^32 elements");
    if ((L + 2048) * (int64_t)shape->d_k * 2 > 0xffffffffLL)
        return fail(LOOKAT_ERR_UNSUPPORTED, "L=%lld: one (b,h) value slab must stay below 4 GiB", (long long)L);
    const int64_t BH = (int64_t)shape->B * shape->H;
    const FlatPlan g = plan_flat(BH, L, num_splits);
    const size_t need = flat_workspace_bytes(BH, shape->d_k, g);
    unsigned *ticket_mem = nullptr;
    float *part_mem = nullptr;
    if (need) {   // counters first, then the pieces
        if (!workspace || workspace_bytes < need)
            return fail(LOOKAT_ERR_WORKSPACE, "workspace of %zu bytes needed, got %zu", need, workspace_bytes);
        if (!aligned16(workspace))
            return fail(LOOKAT_ERR_ALIGN, "workspace must be 16-byte aligned");
        ticket_mem = static_cast<unsigned *>(workspace);
        part_mem = reinterpret_cast<float *>(static_cast<char *>(workspace) + flat_ticket_bytes(BH));
    }
    if (BH * g.tpu + g.share > 0x7fffffffLL || g.shares > 0x7fffffffLL || shape->H > 0xffff)
        return fail(LOOKAT_ERR_UNSUPPORTED, "B*H*tiles=%lld (in %lld workgroups, H=%d) exceed one launch",
                    (long long)(BH * g.tpu), (long long)g.shares, shape->H);
    const FastDiv dt = fastdiv_of((uint32_t)g.tpu);
    const uint32_t H_sh = (uint32_t)shape->H | (dt.sh1 << 16) | (dt.sh2 << 17);
    FlatLate late;
    late.part = part_mem;
    late.tickets = ticket_mem;
    late.out = out;
    late.scores_out = scores_out;
    late.slots = (int)g.slots;
    late.scale_log2e = scale * kLog2e;
    const int waves = flat_waves(shape->d_k, g);
    const size_t lds = ((size_t)kFlatPieces * shape->m * kCentroids + (size_t)kFlatPieces * waves * (shape->d_k + 2)) * sizeof(float) +
                       kFlatPieces * sizeof(unsigned);
    dim3 grid((unsigned)g.shares);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const __half *vh = static_cast<const __half *>(values);
    const uint32_t cs = (uint32_t)code_stride_bh, vs = (uint32_t)value_stride_bh;
    const uint32_t nflat = (uint32_t)(BH * g.tpu), share = (uint32_t)g.share;
#define LOOKAT_FLAT_DK(DK_)                                                                                            \
case DK_:                                                                                                          \
    if (waves == 16)                                                                                               \
        launch_flat<DK_, 16, 0>(shape->m, grid, lds, st, nflat, share, dt.magic, H_sh, lut, codes, vh, cs, vs, (uint32_t)L, late); \
    else if (g.share > g.tpu) /* several pieces per workgroup: a wavefront of its own finishes them */ \
        launch_flat<DK_, 8, 1>(shape->m, grid, lds, st, nflat, share, dt.magic, H_sh, lut, codes, vh, cs, vs, (uint32_t)L, late); \
    else                                                                                                           \
        launch_flat<DK_, 8, 0>(shape->m, grid, lds, st, nflat, share, dt.magic, H_sh, lut, codes, vh, cs, vs, (uint32_t)L, late); \
    break;
    switch (shape->d_k) {
        LOOKAT_FLAT_DK(32)
        LOOKAT_FLAT_DK(64)
        LOOKAT_FLAT_DK(128)
        LOOKAT_FLAT_DK(256)
    }
#undef LOOKAT_FLAT_DK
    if (pieces_per_unit)
        *pieces_per_unit = (int32_t)g.slots;
    return check_launch("lookat_probe_attend_decode_ticket");
}
