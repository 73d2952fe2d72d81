// Loops 2-4 of Algorithm 1 (Lavin & Gray) in one kernel, fp32 F(4x4,3x3) and F(2x2,3x3) (the algorithm of the
// paper's own fused kernel, Section 6), for layers with more than 32 filters.  Described for F(4x4,3x3):
// the design of fused_lds.hip with twice the filters per transformed tile.  On this chip fp32 MFMAs and ordinary
// vector instructions of one SIMD share an issue slot, so the arithmetic of the data transform is paid in MFMA
// time; it is needed once per (tile, channel) and workgroup, whatever the number of filters the workgroup
// multiplies the result with.
//
// Workgroup = 4 wavefronts owning 64 filters x 16 tiles x 36 components (144 accumulators per lane), two per CU.
// Per step of 16 channels:
//   1. transform phase: every thread owns one (tile, channel) pair; taps as in fused_lds.hip (buffer loads one
//      step ahead, out-of-range markers for the implicit zero padding of Section 6), except that a tile's outer
//      columns come from the registers of the neighbouring lanes (DPP) instead of from memory: requests of 4 bytes
//      per lane at a stride of 16 bytes cost the vector memory path as much as the 16-byte ones next to them, and
//      without them the kernel runs a tenth faster; v = B^T (d B) goes to one of two LDS buffers as
//      [e][channel][tile], so there is one barrier per step;
//   2. multiply phase: wavefront cg owns components 9 cg .. 9 cg + 8 and walks four sub-steps of 4 channels
//      (the depth of v_mfma_f32_16x16x4_f32).  The transformed filters do not pass through LDS (64 filters x
//      16 channels x 36 components would fill it): lane (i, h) fetches U[e][channel h of the sub-step][filters
//      4 i .. 4 i + 3] with one 16-byte buffer load, the A operands of the component's four MFMAs (MFMA f takes
//      filter 4 i + f as its row i), and requests the same component of the next sub-step right after these
//      MFMAs: nine components of MFMAs ahead of its use, in the register it replaces.
// After the last step the accumulators go through LDS in four pieces (piece f = the filters 4 i + f); every thread
// gathers the 36 components of one (filter, tile) pair, applies Y = A^T m A and writes its rows.
// Needs pad = 1, W % m == 0 and the images one workgroup touches within 1 GiB.
//
// The resident workgroups (512; 768 for F(2x2)) take the items of their XCD round by round.  A last round that fills
// only part of them would leave most CUs idle for the length of an item, so its items are cut into shares of their channel
// steps, one workgroup per share: each share applies the (linear) inverse transform to its partial sums, stores
// partial outputs in the workspace and takes a ticket; the share that arrives last adds the partial outputs in
// share order and writes Y.  Nobody waits for anybody, and the result does not depend on the order of arrival.
#include <type_traits>

#include "wino_internal.h"
#include "transforms.h"

namespace wino {

typedef float floatx4_w __attribute__((ext_vector_type(4)));

constexpr int FW_K = 64, FW_P = 16, FW_C = 16, FW_T = 256;          // filters, tiles, channels per step, threads
constexpr int fw_v_floats(int m) { return (m + 2) * (m + 2) * FW_C * FW_P; }   // transformed tiles of a step (one buffer)
constexpr int fw_m_floats(int m) { return (m + 2) * (m + 2) * 16 * 16; }       // one piece of M in the epilogue: [e][filter row][tile]
constexpr unsigned FW_MAX_BYTES = 0x40000000u;                      // longest stretch of D one workgroup's buffer covers
constexpr unsigned FW_ROW_OOB = 0x80000000u, FW_COL_OOB = 0x40000000u;   // offset markers of taps outside the image
static_assert(fw_m_floats(4) <= 2 * fw_v_floats(4) && fw_m_floats(2) <= 2 * fw_v_floats(2), "the epilogue reuses the two tile buffers");
// Resident workgroups: registers and LDS allow two per CU for F(4x4) and three for F(2x2) (145 registers, 32 KB).
constexpr int fw_per_cu(int m) { return m == 4 ? 2 : 3; }
constexpr int fw_grid(int m) { return 256 * fw_per_cu(m); }
constexpr int fw_share_floats(int m) { return FW_K * FW_P * m * m; }       // partial outputs of one share
constexpr int FW_TICKETS = 1024;                                    // arrival counters in front of the partial outputs
constexpr int FW_TICKET_BYTES = FW_TICKETS * 4;
static_assert(fw_grid(4) <= FW_TICKETS && fw_grid(2) <= FW_TICKETS, "one counter per resident workgroup at most");

// The items an XCD's workgroups walk (`count` of them, `slots` workgroups): `full` items in rounds that occupy
// every workgroup, then `tail` items cut into `shares` shares of their `nsteps` channel steps each.  Items of
// fewer than 16 steps are not shared, nor are items that could only be halved: the workgroups of a partly filled
// round have their CUs to themselves and run 1.7 times faster for it, and the hand-over costs about 10 us
// (measured at batch 64: 256 channels and more gain 2-9 % per layer, 64 and 128 channels lose 1.5 %).
struct FwRounds {
    int full, tail, shares;
};
__host__ __device__ inline FwRounds fw_rounds(int count, int slots, int nsteps, bool may_share)
{
    FwRounds r;
    r.full = may_share && nsteps >= 16 ? count / slots * slots : count;
    r.tail = count - r.full;
    r.shares = 1;
    while (r.tail > 0 && r.shares < 8 && r.shares * 2 * r.tail <= slots && nsteps % (r.shares * 2) == 0) r.shares *= 2;
    if (r.shares < 4) r.full = count, r.tail = 0, r.shares = 1;      // the last round runs whole items
    return r;
}
// Items of XCD `xcd`: [first, first + count) of its group's list (see the kernel).
__host__ __device__ inline void fw_list(int xcd, int groups, int n_kb, int n_tb, int *first, int *count)
{
    const int member = xcd / groups, members = 8 / groups;
    const int group_items = n_tb * (n_kb / groups);
    const int per_member = (group_items + members - 1) / members;
    const int end = (member + 1) * per_member < group_items ? (member + 1) * per_member : group_items;
    *first = member * per_member;
    *count = end > *first ? end - *first : 0;
}

// Partial outputs pass between workgroups that may sit on different XCDs, whose L2 caches are not coherent with
// each other: they are written and read with agent-scope atomic accesses (relaxed, 8 bytes), which go through to
// the level all XCDs share.  A store counts in the wavefront's vmcnt until that level has acknowledged it, so
// every wavefront waits for vmcnt(0) before the barrier that precedes the ticket (see fused_f2.hip).
typedef float floatx2_w __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void fw_st_agent(float *p, float a, float b)
{
    const floatx2_w v = {a, b};
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), __builtin_bit_cast(unsigned long long, v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ floatx2_w fw_ld_agent(const float *p)
{
    const unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
    return __builtin_bit_cast(floatx2_w, u);
}

// Position of filter row r (0..15) within a component of a piece of M.  Rows are 16 floats, so two rows of equal
// parity share their banks; a wavefront writes rows r and r + 4 together and reads rows r and r + 1 together, and
// with this permutation both pairs differ in parity.
__device__ __forceinline__ int fw_m_row(int r) { return r ^ ((r >> 2) & 1); }

// Barrier that orders LDS traffic only: global loads requested earlier stay in flight across it.
__device__ __forceinline__ void fw_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// The M x M outputs of one (filter, tile) pair: whole rows of 16 (F(4x4)) or 8 bytes (F(2x2)), not kept in the caches;
// `rows` = rows of the image left from the tile's first one.
template <int M>
__device__ __forceinline__ void fw_store_rows(float *dst, int Wo, int rows, const float (&y)[M][M])
{
#pragma unroll
    for (int p = 0; p < M; ++p)
        if (p < rows) {
            if constexpr (M == 4)
                __builtin_nontemporal_store(floatx4_w{y[p][0], y[p][1], y[p][2], y[p][3]},
                                            reinterpret_cast<floatx4_w *>(dst + (size_t)p * Wo));
            else
                __builtin_nontemporal_store(floatx2_w{y[p][0], y[p][1]}, reinterpret_cast<floatx2_w *>(dst + (size_t)p * Wo));
        }
}

// M: F(M x M, 3 x 3), 4 or 2 (the comments name the numbers of F(4x4): 6 x 6 tiles, 36 components, 9 per wavefront;
// F(2x2) has 4 x 4, 16 and 4, its rows are 8-byte loads and stores).
// CPAD: the channel count is not a multiple of 16, so the last step holds channel slots past the last channel.
template <int M, bool CPAD>
__global__ __launch_bounds__(FW_T, fw_per_cu(M)) void fused_wide_kernel(const float *__restrict__ D, const float *__restrict__ U,
                                                             float *__restrict__ Y, Geo g, int n_kb, int n_tb, int groups,
                                                             float *__restrict__ part)
{
    constexpr int A = M + 2, NE = A * A, EW = NE / 4;          // tile edge, components, components per wavefront
    constexpr int FW_V_FLOATS = fw_v_floats(M);
    typedef float mid_t __attribute__((ext_vector_type(M)));   // the M middle columns of a tile row
    __shared__ __attribute__((aligned(16))) float smem[2 * FW_V_FLOATS];
    const int tid = threadIdx.x;

    // Resident workgroups walking a list of (tile block, filter block) items (see fused_lds.hip).  The 8 XCDs form
    // `groups` groups; a group takes n_kb / groups of the filter blocks -- as many as keep their transformed filters
    // in one XCD's L2, where every sub-step of every workgroup reads them -- and all tile blocks; its XCDs take
    // one contiguous part of these items each, consecutive items being the filter blocks of one tile block, which
    // read the same input.
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8, slots = gridDim.x / 8;
    const int group = xcd % groups;
    const int kb_per_group = n_kb / groups;
    int first, count;
    fw_list(xcd, groups, n_kb, n_tb, &first, &count);
    // (no shares without a workspace for partial outputs: `part` null)
    const int nsteps_all = (g.C + FW_C - 1) / FW_C;  // U holds zeros for the channels between C and Cp (a multiple of 16)
    const FwRounds rounds = fw_rounds(count, slots, nsteps_all, part != nullptr);
    const int full = rounds.full, tail = rounds.tail, shares = rounds.shares;
    unsigned int *const tickets = reinterpret_cast<unsigned int *>(part);
    float *const partial = part + FW_TICKET_BYTES / 4;
    for (int it = slot;; it += slots) {
    int item, step0 = 0, nsteps = nsteps_all;
    bool shared = false;
    if (it < full) {
        item = first + it;
    } else if (it - full < tail * shares) {
        item = first + full + (it - full) % tail;
        shared = true;
        nsteps = nsteps_all / shares;
        step0 = (it - full) / tail * nsteps;
    } else {
        break;
    }
    const int kb = group * kb_per_group + item % kb_per_group, tb = item / kb_per_group;
    const int k0 = kb * FW_K, b0 = tb * FW_P;

    // ---- transform-phase role: (tile, channel slot of the step) ---------------------------------
    const int tl = tid & 15, cl = tid >> 4;
    const int b = b0 + tl;
    const bool tile_ok = b < g.P;
    int orow = 0;
    float *ybase = Y;
    const int tiles_per_image = g.Th * g.Tw;
    const int img0 = b0 / tiles_per_image;                     // uniform
    unsigned vo_m[A];                                          // byte offset of columns 1..4 of row p, channel slot cl, step 0
    // The outer columns (0 and 5) of a tile are column 4 of the tile to its left and column 1 of the tile to its
    // right.  The 16 tiles of the workgroup sit in the 16 lanes of a DPP row, so a lane takes them from its
    // neighbours' registers; only the first lane of a row lacks its left neighbour and the last lane its right one.
    // Those twelve values per step (six tile rows each) are fetched by ONE request in which lanes 1..6 of the row
    // ask for the first lane's left column of tile rows 0..5 and lanes 8..13 for the last lane's right column
    // (`edge_off`; a marker in the other lanes), and handed over by DPP as well.  A tile at the image's left or
    // right border has zeros there (`left_in`, `right_in`), whatever its neighbour lane holds: the last tile of the
    // tile row above, or the first of the one below.
    unsigned edge_off;
    bool left_in, right_in;
    {
        const int bb = tile_ok ? b : b0;
        const int ty = bb % g.Tw;
        const int t2 = bb / g.Tw;
        const int tx = t2 % g.Th;
        const int i = t2 / g.Th;
        const int x0 = M * tx - 1, y0 = M * ty - 1;
        orow = M * tx;
        ybase = Y + ((size_t)i * g.K * g.Ho + orow) * g.Wo + M * ty;
        left_in = y0 >= 0;
        right_in = y0 + A - 1 < g.W;
        const unsigned plane0 = (unsigned)((i - img0) * g.C + cl) * (unsigned)(g.H * g.W);
#pragma unroll
        for (int p = 0; p < A; ++p) {
            const int x = x0 + p;
            const bool rok = tile_ok && x >= 0 && x < g.H;
            vo_m[p] = rok ? (plane0 + (unsigned)(x * g.W + y0 + 1)) * 4u : FW_ROW_OOB;   // column y0 + 1 = M ty
        }
        // Every lane forms the offsets of its own outer columns (marked where they lie outside the image); lane
        // 1 + p then takes the left one of tile row p from the first lane of its DPP row and lane 8 + p the right
        // one from the last lane.  A shift by n also reaches the lanes further on: the left chain runs with n
        // rising and the right chain with n falling, so that the value from the end lane is the last one a lane
        // receives.
        const unsigned adj_l = left_in ? 0xfffffffcu /* -4 bytes */ : FW_COL_OOB, adj_r = right_in ? 4u * M : FW_COL_OOB;
        int from_first = (int)FW_COL_OOB, from_last = (int)FW_COL_OOB;
        from_first = __builtin_amdgcn_update_dpp(from_first, (int)(vo_m[0] + adj_l), 0x111, 0xf, 0xf, false);   // row_shr:1
        from_first = __builtin_amdgcn_update_dpp(from_first, (int)(vo_m[1] + adj_l), 0x112, 0xf, 0xf, false);
        from_first = __builtin_amdgcn_update_dpp(from_first, (int)(vo_m[2] + adj_l), 0x113, 0xf, 0xf, false);
        from_first = __builtin_amdgcn_update_dpp(from_first, (int)(vo_m[3] + adj_l), 0x114, 0xf, 0xf, false);
        if constexpr (M == 4) {
            from_first = __builtin_amdgcn_update_dpp(from_first, (int)(vo_m[A - 2] + adj_l), 0x115, 0xf, 0xf, false);
            from_first = __builtin_amdgcn_update_dpp(from_first, (int)(vo_m[A - 1] + adj_l), 0x116, 0xf, 0xf, false);
            from_last = __builtin_amdgcn_update_dpp(from_last, (int)(vo_m[A - 1] + adj_r), 0x102, 0xf, 0xf, false);     // row_shl:2
            from_last = __builtin_amdgcn_update_dpp(from_last, (int)(vo_m[A - 2] + adj_r), 0x103, 0xf, 0xf, false);
        }
        from_last = __builtin_amdgcn_update_dpp(from_last, (int)(vo_m[3] + adj_r), 0x104, 0xf, 0xf, false);
        from_last = __builtin_amdgcn_update_dpp(from_last, (int)(vo_m[2] + adj_r), 0x105, 0xf, 0xf, false);
        from_last = __builtin_amdgcn_update_dpp(from_last, (int)(vo_m[1] + adj_r), 0x106, 0xf, 0xf, false);
        from_last = __builtin_amdgcn_update_dpp(from_last, (int)(vo_m[0] + adj_r), 0x107, 0xf, 0xf, false);
        edge_off = (tl >= 1 && tl <= A) ? (unsigned)from_first : (tl >= 8 && tl <= 7 + A) ? (unsigned)from_last : FW_COL_OOB;
    }
    const unsigned step_bytes = (unsigned)(FW_C * g.H * g.W) * 4u;
    const size_t image_floats = (size_t)g.C * g.H * g.W;
    const size_t left = ((size_t)g.N - img0) * image_floats * 4;
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(D + (size_t)img0 * image_floats), 0, (unsigned)(left < FW_MAX_BYTES ? left : FW_MAX_BYTES), 0x00020000);
    const __amdgpu_buffer_rsrc_t rsrc_u =
        __builtin_amdgcn_make_buffer_rsrc((void *)U, 0, (unsigned)((size_t)NE * g.Cp * g.Kp * 4), 0x00020000);

    // ---- multiply-phase role -------------------------------------------------------------------
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int cg = wave;
    const int lj = lane & 15, lk = lane >> 4;
    floatx4_w acc[EW][4];
#pragma unroll
    for (int e = 0; e < EW; ++e)
#pragma unroll
        for (int f = 0; f < 4; ++f) acc[e][f] = floatx4_w{0.0f, 0.0f, 0.0f, 0.0f};

    // A operands: U[((9 cg + e) Cp + 4 sub + lk) Kp + k0 + 4 lj .. + 3], sub = 4 step + sub-step.  Where the
    // filter block reaches past Kp the last four columns are read instead: rows of filters that are never stored.
    const unsigned uvo = (unsigned)(lk * g.Kp + min(k0 + 4 * lj, g.Kp - 4)) * 4u;
    const unsigned ue_bytes = (unsigned)(g.Cp * g.Kp) * 4u, usub_bytes = (unsigned)(4 * g.Kp) * 4u;
    unsigned su = (unsigned)(cg * EW) * ue_bytes + (unsigned)(4 * step0) * usub_bytes;      // scalar offset of component 9 cg in the sub-step requested next
    // KC sub-steps of filter operands are in flight: one for F(4x4) (nine components of MFMAs, 1152 cycles, ahead of
    // their use), two for F(2x2), whose sub-step has only four components
    constexpr int KC = M == 4 ? 1 : 2;
    floatx4_w ua[KC * EW];
    auto load_ua = [&](int slot, int e, unsigned vo) {
        ua[slot] = __builtin_bit_cast(floatx4_w, __builtin_amdgcn_raw_buffer_load_b128(rsrc_u, vo, su + e * ue_bytes, 0));
    };
    mid_t mid[A];
    float ed;
    // `valid` false: nothing is fetched (every offset is a marker).  The request is made all the same, so that the
    // number of loads in flight does not depend on the path taken (the compiler's wait counts take the minimum).
    auto load_taps = [&](int step, bool valid) {
        const unsigned so = valid ? (unsigned)step * step_bytes : 0u;
        // (an OR with a uniform mask, not a choice between two offsets: the compiler turns the latter into a branch
        // around two load instructions, and behind the join it waits for every request in flight)
        const unsigned off_mask = valid ? 0u : FW_ROW_OOB;
        const bool ch_ok = !CPAD || (step * FW_C + cl < g.C);
#pragma unroll
        for (int p = 0; p < A; ++p) {
            const unsigned om = (ch_ok ? vo_m[p] : FW_ROW_OOB) | off_mask;
            if constexpr (M == 4)
                mid[p] = __builtin_bit_cast(mid_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc, om, so, 0));
            else
                mid[p] = __builtin_bit_cast(mid_t, __builtin_amdgcn_raw_buffer_load_b64(rsrc, om, so, 0));
        }
        ed = __builtin_bit_cast(float,
                                __builtin_amdgcn_raw_buffer_load_b32(rsrc, (ch_ok ? edge_off : FW_ROW_OOB) | off_mask, so, 0));
    };
    // this thread's tile: rows then columns (v = B^T (d B)), scatter to LDS buffer `buf` as [e][channel][tile]
    auto transform = [&](int buf) {
        float t[A][A];
        // tile row p (a compile-time constant: it selects the DPP shifts)
        auto row = [&](auto pc) {
            constexpr int p = decltype(pc)::value;
            // column 4 of the lane below (row_shr:1), column 1 of the lane above (row_shl:1); the first and the last
            // lane of the row, which have no such neighbour, keep what lane 1 + p resp. 8 + p fetched for them
            const float c1 = mid[p][0], c4 = mid[p][M - 1];  // (a bit cast applied to a vector element would read element 0)
            const int e_bits = __builtin_bit_cast(int, ed);
            // (lanes without a source lane read 0: only the first resp. the last lane's value is used)
            const int for_first = __builtin_amdgcn_mov_dpp(e_bits, 0x101 + p, 0xf, 0xf, true);   // row_shl:(1 + p)
            const int for_last = __builtin_amdgcn_mov_dpp(e_bits, 0x117 - p, 0xf, 0xf, true);    // row_shr:(7 - p)
            const int l_bits = __builtin_amdgcn_update_dpp(for_first, __builtin_bit_cast(int, c4), 0x111, 0xf, 0xf, false);
            const int r_bits = __builtin_amdgcn_update_dpp(for_last, __builtin_bit_cast(int, c1), 0x101, 0xf, 0xf, false);
            const float lv = left_in ? __builtin_bit_cast(float, l_bits) : 0.0f;
            const float rv = right_in ? __builtin_bit_cast(float, r_bits) : 0.0f;
            float d[A];
            d[0] = lv, d[A - 1] = rv;
#pragma unroll
            for (int q = 0; q < M; ++q) d[1 + q] = mid[p][q];
            bt_mul<M>(d, t[p]);
        };
        row(std::integral_constant<int, 0>());
        row(std::integral_constant<int, 1>());
        row(std::integral_constant<int, 2>());
        row(std::integral_constant<int, 3>());
        if constexpr (M == 4) {
            row(std::integral_constant<int, A - 2>());
            row(std::integral_constant<int, A - 1>());
        }
        float *dst = smem + buf * FW_V_FLOATS + tid;       // cl * 16 + tl = tid
#pragma unroll
        for (int q = 0; q < A; ++q) {
            float col[A], o[A];
#pragma unroll
            for (int p = 0; p < A; ++p) col[p] = t[p][q];
            bt_mul<M>(col, o);
#pragma unroll
            for (int p = 0; p < A; ++p) dst[(p * A + q) * (FW_C * FW_P)] = o[p];
        }
    };
    // nine components x four sub-steps x (64 filters x 16 tiles x 4 channels); B operand of lane (j, h) in
    // sub-step t: channel 4 t + h of tile j, i.e. float e * 256 + t * 64 + lane of the buffer.
    auto multiply = [&](int buf, bool more) {
        // the next step's first sub-step is requested during the last sub-step of this one (in flight over the
        // transform phase); with no next step the request is made with an offset behind the buffer, which fetches
        // nothing, so that the number of loads in flight does not depend on the path taken
        const unsigned uvo_next = more ? uvo : 0x80000000u;
        const float *vb = smem + buf * FW_V_FLOATS + cg * EW * (FW_C * FW_P) + lane;
        float bq[2];
        bq[0] = vb[0];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
#pragma unroll
            for (int e = 0; e < EW; ++e) {
                const int n = t * EW + e, slot = (t % KC) * EW + e;
                if (n + 1 < 4 * EW) bq[(n + 1) & 1] = vb[((n + 1) % EW) * (FW_C * FW_P) + ((n + 1) / EW) * 64];
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int f = 0; f < 4; ++f)
                    acc[e][f] = __builtin_amdgcn_mfma_f32_16x16x4f32(ua[slot][f], bq[n & 1], acc[e][f], 0, 0, 0);
                load_ua(slot, e, t + KC < 4 ? uvo : uvo_next);      // the same component KC sub-steps on
                __builtin_amdgcn_sched_barrier(0);
            }
            su += usub_bytes;
        }
    };

    // One iteration = transform phase of a step, then its multiply phase; the taps a transform phase consumes were
    // requested in the iteration before (first: here), right after the barrier, when their registers came free.
    load_taps(step0, true);
    // (kept in this order: were the filter requests moved ahead of the taps, the wait for the taps at the top of
    // the loop -- which the compiler derives from both ways into it -- would also end the filter requests' flight)
    __builtin_amdgcn_sched_barrier(0x38f);        // everything but memory requests may cross
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
#pragma unroll
        for (int e = 0; e < EW; ++e) load_ua(kc * EW + e, e, uvo);
        su += usub_bytes;
    }
    for (int step = 0; step < nsteps; ++step) {
        const int buf = step & 1;
        const bool more = step + 1 < nsteps;
        // A wavefront in its transform phase or epilogue shares its SIMD with one of the other workgroup, which
        // as a rule is issuing MFMAs; at equal priority the two take turns, one vector instruction per MFMA (the
        // 100 vector instructions of an epilogue piece take 3 500 cycles that way).  With the higher priority here
        // the phase passes quickly and the wavefront is back at its own MFMAs sooner: 2-3 % per layer.
        __builtin_amdgcn_s_setprio(3);
        transform(buf);
        __builtin_amdgcn_s_setprio(0);
        fw_lds_barrier();
        load_taps(step0 + step + 1, more);
        multiply(buf, more);
    }
    __builtin_amdgcn_s_setprio(2);
    __syncthreads();

    // ---- inverse transform: four pieces of 16 filters (piece f = filters k0 + 4 i + f, i = 0..15) ----------
    constexpr int NJ = M * M / 2;              // pairs of outputs per (filter, tile)
    float *Ms = smem;
    const int irow = tid >> 4;                 // 0..15: filter row of the piece handled in the gather
    const int ot = tid & 15;                   // tile of the gather (same tile as in the transform phase)
#pragma unroll
    for (int f = 0; f < 4; ++f) {
        // accumulator register rr of lane (lj, lk) is row 4 lk + rr, tile lj
#pragma unroll
        for (int e = 0; e < EW; ++e)
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) Ms[((cg * EW + e) * 16 + fw_m_row(4 * lk + rr)) * 16 + lj] = acc[e][f][rr];
        __syncthreads();
        const int k = k0 + 4 * irow + f;
        if (tile_ok && k < g.K) {
            float m[A][A], tt[M][A], y[M][M];
#pragma unroll
            for (int xi = 0; xi < A; ++xi)
#pragma unroll
                for (int nu = 0; nu < A; ++nu) m[xi][nu] = Ms[((xi * A + nu) * 16 + fw_m_row(irow)) * 16 + ot];
#pragma unroll
            for (int nu = 0; nu < A; ++nu) {
                float col[A], o[M];
#pragma unroll
                for (int xi = 0; xi < A; ++xi) col[xi] = m[xi][nu];
                at_mul<M>(col, o);
#pragma unroll
                for (int p = 0; p < M; ++p) tt[p][nu] = o[p];
            }
#pragma unroll
            for (int p = 0; p < M; ++p) at_mul<M>(tt[p], y[p]);
            if (!shared) {
                fw_store_rows<M>(ybase + (size_t)k * g.Ho * g.Wo, g.Wo, g.Ho - orow, y);
            } else {
                // partial outputs of this share: [piece f][pair j of a row][thread] pairs of floats
                float *dst = partial + (size_t)(xcd * slots + (it - full)) * fw_share_floats(M) + (f * NJ * FW_T + tid) * 2;
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    fw_st_agent(dst + j * FW_T * 2, y[j / (M / 2)][2 * (j % (M / 2))], y[j / (M / 2)][2 * (j % (M / 2)) + 1]);
            }
        }
        __syncthreads();
    }
    __builtin_amdgcn_s_setprio(0);
    if (shared) {
        // ---- the share that arrives last adds the partial outputs of all shares, in share order ----
        const int j_item = (it - full) % tail;
        unsigned int *const ticket = &tickets[xcd * slots + j_item];
        __builtin_amdgcn_s_waitcnt(0x0f70);       // vmcnt(0): this wavefront's partial outputs have been acknowledged ...
        __syncthreads();                          // ... and so have those of the other three
        int *const s_last = reinterpret_cast<int *>(smem);
        if (tid == 0)
            *s_last = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(shares - 1);
        __syncthreads();
        const bool last = *s_last != 0;
        __syncthreads();                          // (smem is written again by the next item)
        if (last) {
            // two shares (64 loads per thread for F(4x4)) in flight at a time; the sums run over the shares in order
            floatx2_w y2[4][NJ];
#pragma unroll
            for (int f = 0; f < 4; ++f)
#pragma unroll
                for (int j = 0; j < NJ; ++j) y2[f][j] = floatx2_w{0.0f, 0.0f};
            const float *src0 = partial + (size_t)(xcd * slots + j_item) * fw_share_floats(M) + tid * 2;
            for (int z = 0; z < shares; z += 2) {
                floatx2_w v[2][4][NJ];
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int f = 0; f < 4; ++f)
#pragma unroll
                        for (int j = 0; j < NJ; ++j)
                            v[h][f][j] = fw_ld_agent(src0 + (size_t)((z + h) * tail) * fw_share_floats(M) + (f * NJ + j) * FW_T * 2);
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int f = 0; f < 4; ++f)
#pragma unroll
                        for (int j = 0; j < NJ; ++j) y2[f][j] += v[h][f][j];
            }
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const int k = k0 + 4 * irow + f;
                if (tile_ok && k < g.K) {
                    float y[M][M];
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        y[j / (M / 2)][2 * (j % (M / 2))] = y2[f][j][0];
                        y[j / (M / 2)][2 * (j % (M / 2)) + 1] = y2[f][j][1];
                    }
                    fw_store_rows<M>(ybase + (size_t)k * g.Ho * g.Wo, g.Wo, g.Ho - orow, y);
                }
            }
        }
    }
    }   // items
}

bool fused_wide_eligible(const Geo &g)
{
    // the tiles of one workgroup span at most `span` images; their byte offsets from the first must stay below 2^30
    const unsigned long long tiles = (unsigned long long)g.Th * g.Tw;
    const unsigned long long span = (FW_P + tiles - 2) / tiles + 1;
    const unsigned long long image_bytes = (unsigned long long)g.C * g.H * g.W * 4ull;
    return g.dt == WINO_F32 && (g.m == 4 || g.m == 2) && g.pad == 1 && g.W % g.m == 0 && g.Kp >= FW_K &&
           span * image_bytes + 65536 < FW_MAX_BYTES &&
           (unsigned long long)g.a2 * g.Cp * g.Kp * 4ull < (1ull << 31);   // 32-bit byte offsets into U
}

// XCD groups: halve the filter blocks per group while their transformed filters (alpha^2 x Cp x 64 floats each) exceed
// what an XCD's 4 MB L2 can keep next to the streams of input and output (measured at N = 64: reads from
// beyond L2 fall from 427 to 325 MB for 128 -> 256 channels at 56 x 56, from 1291 to 1028 MB for 256 -> 256,
// at equal run time).
static int fw_groups(const Geo &g, int n_kb)
{
    int groups = 1;
    while (groups < 8 && n_kb % (2 * groups) == 0 &&
           (unsigned long long)(n_kb / groups) * g.a2 * g.Cp * FW_K * 4 > (5ull << 19))
        groups *= 2;
    return groups;
}

// How well the rounds of a launch are filled: items per workgroup / rounds the slowest XCD takes, a last round
// costing 1 / shares + 0.2 rounds when shared, else 0.6 rounds up to half full (its workgroups alone on their
// CUs) and a whole one beyond (a model of the measurements quoted in fused_preferred).
double fused_wide_fill(const Geo &g)
{
    const int n_kb = (g.Kp + FW_K - 1) / FW_K;
    const long long n_tb = (g.P + FW_P - 1) / FW_P;
    const int full_grid = fw_grid(g.m);
    if (n_tb * n_kb < full_grid || n_tb * n_kb > 0x7fffffffLL) return 0.0;
    const int groups = fw_groups(g, n_kb), slots = full_grid / 8, nsteps = (g.C + FW_C - 1) / FW_C;
    double worst = 0.0;
    for (int xcd = 0; xcd < 8; ++xcd) {
        int first, count;
        fw_list(xcd, groups, n_kb, (int)n_tb, &first, &count);
        const FwRounds r = fw_rounds(count, slots, nsteps, true);
        double rounds = (double)(r.full / slots);
        if (r.shares > 1)
            rounds += 1.0 / r.shares + 0.2;
        else if (r.full % slots != 0)
            rounds += r.full % slots * 2 <= slots ? 0.6 : 1.0;
        worst = rounds > worst ? rounds : worst;
    }
    return (double)(n_tb * n_kb) / full_grid / worst;
}

size_t fused_wide_part_bytes(const Geo &g)
{
    return FW_TICKET_BYTES + (size_t)fw_grid(g.m) * fw_share_floats(g.m) * sizeof(float);
}

// Sets the arrival counters to zero (a kernel, not a memset: the launch may be recorded into a graph).
__global__ void fused_wide_clear_kernel(unsigned int *tickets) { tickets[threadIdx.x] = 0u; }

// Shares need the full grid (their places in the workspace and the counters are numbered by it) and room for the
// counters and the partial outputs; otherwise, or where no XCD has a last round to share, whole items.
bool fused_wide_shares(const Geo &g, const void *part, size_t part_bytes)
{
    const int n_kb = (g.Kp + FW_K - 1) / FW_K;
    const long long n_tb = (g.P + FW_P - 1) / FW_P;
    if (part == nullptr || part_bytes < fused_wide_part_bytes(g) || n_tb * n_kb < fw_grid(g.m) || n_tb * n_kb > 0x7fffffffLL)
        return false;
    const int groups = fw_groups(g, n_kb);
    for (int xcd = 0; xcd < 8; ++xcd) {
        int first, count;
        fw_list(xcd, groups, n_kb, (int)n_tb, &first, &count);
        if (fw_rounds(count, fw_grid(g.m) / 8, (g.C + FW_C - 1) / FW_C, true).shares > 1) return true;
    }
    return false;
}

int fused_wide_plan(const Geo &g, int out[32])
{
    const int n_kb = (g.Kp + FW_K - 1) / FW_K;
    const long long n_tb = (g.P + FW_P - 1) / FW_P;
    const long long items = n_tb * n_kb;
    if (items > 0x7fffffffLL) return -1;
    const int groups = fw_groups(g, n_kb);
    const int grid = (int)(items >= fw_grid(g.m) ? fw_grid(g.m) : (items + 7) / 8 * 8);
    for (int xcd = 0; xcd < 8; ++xcd) {
        int first, count;
        fw_list(xcd, groups, n_kb, (int)n_tb, &first, &count);
        const FwRounds r = fw_rounds(count, grid / 8, (g.C + FW_C - 1) / FW_C, grid == fw_grid(g.m));
        out[4 * xcd] = count, out[4 * xcd + 1] = r.full, out[4 * xcd + 2] = r.tail, out[4 * xcd + 3] = r.shares;
    }
    return grid;
}

hipError_t launch_fused_wide(const Geo &g, const float *D, const float *U, float *Y, void *part, size_t part_bytes,
                             bool cleared, hipStream_t s)
{
    const int n_kb = (g.Kp + FW_K - 1) / FW_K;
    const int n_tb = (g.P + FW_P - 1) / FW_P;
    const long long items = (long long)n_tb * n_kb;
    if (items > 0x7fffffffLL) return hipErrorInvalidValue;
    const int groups = fw_groups(g, n_kb);
    // as many workgroups as stay resident on 256 CUs, in multiples of the 8 XCDs
    const unsigned grid = (unsigned)(items >= fw_grid(g.m) ? fw_grid(g.m) : (items + 7) / 8 * 8);
    float *p = fused_wide_shares(g, part, part_bytes) ? (float *)part : nullptr;
    if (p != nullptr && !cleared) fused_wide_clear_kernel<<<dim3(1), dim3(FW_TICKETS), 0, s>>>((unsigned int *)p);
    const bool cpad = g.C % FW_C != 0;
    if (g.m == 4 && cpad)
        fused_wide_kernel<4, true><<<dim3(grid), dim3(FW_T), 0, s>>>(D, U, Y, g, n_kb, n_tb, groups, p);
    else if (g.m == 4)
        fused_wide_kernel<4, false><<<dim3(grid), dim3(FW_T), 0, s>>>(D, U, Y, g, n_kb, n_tb, groups, p);
    else if (cpad)
        fused_wide_kernel<2, true><<<dim3(grid), dim3(FW_T), 0, s>>>(D, U, Y, g, n_kb, n_tb, groups, p);
    else
        fused_wide_kernel<2, false><<<dim3(grid), dim3(FW_T), 0, s>>>(D, U, Y, g, n_kb, n_tb, groups, p);
    return hipGetLastError();
}

}  // namespace wino
